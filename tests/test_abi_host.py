"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching any device."""
import ctypes
import os
import re

import pytest

import paper_2503_20552_amd as adr
from paper_2503_20552_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # non-null, 16-byte aligned, never dereferenced on an error path


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "adr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adr_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = adr.load_library()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert adr.adr_version() >= 100
    assert adr.adr_status_string(0) == "ok"
    assert "unknown" in adr.adr_status_string(99)


def cache(**kw):
    c = dict(k=FAKE, v=FAKE, k_scale=None, v_scale=None, num_pages=8, page_size=16, Hkv=2, d=128,
             dtype=adr.ADR_BF16)
    c.update(kw)
    return binding._CCache(*[c[f] for f, _ in binding._CCache._fields_])


def attention(c, **kw):
    a = dict(out=FAKE, out_dtype=adr.ADR_BF16, lse=None, q=FAKE, q_row_stride=8 * 128, cache=c,
             block_table=FAKE, max_pages=4, seq_lens=FAKE, B=2, Hq=8, scale=0.1, max_seq_len=64,
             partition_tokens=0, workspace=None, workspace_bytes=0, flags=0, stream=None)
    a.update(kw)
    lib = adr.load_library()
    return lib.adr_decode_attention(a["out"], a["out_dtype"], a["lse"], a["q"], a["q_row_stride"],
                                    ctypes.byref(a["cache"]), a["block_table"], a["max_pages"],
                                    a["seq_lens"], a["B"], a["Hq"], a["scale"], a["max_seq_len"],
                                    a["partition_tokens"], a["workspace"], a["workspace_bytes"],
                                    a["flags"], a["stream"])


NULL, SHAPE, UNSUP, WORK = 1, 2, 3, 4


@pytest.mark.parametrize("kw,expect", [
    (dict(out=None), NULL), (dict(q=None), NULL), (dict(block_table=None), NULL),
    (dict(seq_lens=None), NULL),
    (dict(Hq=7), SHAPE),                       # not a multiple of Hkv
    (dict(q_row_stride=8 * 128 - 8), SHAPE),   # rows overlap
    (dict(q_row_stride=8 * 128 + 4), SHAPE),   # rows lose 16-byte alignment
    (dict(q=FAKE + 2), SHAPE), (dict(out=FAKE + 8), SHAPE),
    (dict(max_seq_len=65), SHAPE),             # more tokens than the table can name
    (dict(partition_tokens=24), SHAPE),        # not a multiple of the page size
    (dict(partition_tokens=-16), SHAPE),
    (dict(B=-1), SHAPE),
    (dict(out_dtype=adr.ADR_FP8_E4M3), UNSUP),
    (dict(flags=4), UNSUP), (dict(flags=256), UNSUP), (dict(flags=1 << 28), UNSUP),
    (dict(Hq=2 * 32, q_row_stride=64 * 128), UNSUP),   # G = 32
    (dict(partition_tokens=16), WORK),         # split needs a workspace
    (dict(partition_tokens=16, workspace=FAKE, workspace_bytes=16), WORK),
    (dict(partition_tokens=16, workspace=FAKE + 16, workspace_bytes=1 << 30), WORK),  # misaligned
])
def test_decode_attention_rejects_bad_arguments(kw, expect):
    assert attention(cache(), **kw) == expect


@pytest.mark.parametrize("kw,expect", [
    (dict(k=None), NULL), (dict(v=None), NULL), (dict(num_pages=0), SHAPE), (dict(Hkv=0), SHAPE),
    (dict(page_size=48), UNSUP), (dict(page_size=128), UNSUP), (dict(d=96), UNSUP), (dict(dtype=adr.ADR_F32), UNSUP),
    (dict(dtype=adr.ADR_FP8_E4M3), NULL),      # fp8 without scales
    (dict(k=FAKE + 4), SHAPE),
])
def test_cache_descriptor_is_validated(kw, expect):
    assert attention(cache(**kw)) == expect


def test_pages_of_32_and_64_tokens_are_accepted_and_bound_the_partition_size():
    assert attention(cache(page_size=32), B=0) == 0 and attention(cache(page_size=64), B=0) == 0
    assert attention(cache(page_size=32), partition_tokens=48) == SHAPE      # not a multiple of the page size
    assert attention(cache(page_size=32), max_seq_len=129) == SHAPE          # 4 pages name 128 tokens
    assert attention(cache(page_size=32), max_seq_len=128, B=0) == 0


def test_mfma_only_for_d128_and_valu_only_for_small_groups():
    assert attention(cache(d=64), flags=adr.KERNEL_MFMA) == UNSUP
    assert attention(cache(Hkv=1), Hq=16, flags=adr.KERNEL_VALU, q_row_stride=16 * 128) == UNSUP


def test_empty_batch_is_ok_without_launch():
    assert attention(cache(), B=0) == 0


def test_append_rejects_bad_arguments():
    lib = adr.load_library()
    c = cache()

    def call(**kw):
        a = dict(k_new=FAKE, v_new=FAKE, stride=2 * 128, bt=FAKE, max_pages=4, pos=FAKE, B=2)
        a.update(kw)
        return lib.adr_kv_append(ctypes.byref(c), a["k_new"], a["v_new"], a["stride"], a["bt"],
                                 a["max_pages"], a["pos"], a["B"], None)
    assert call(k_new=None) == NULL and call(pos=None) == NULL and call(bt=None) == NULL
    assert call(stride=128) == SHAPE and call(stride=2 * 128 + 2) == SHAPE
    assert call(max_pages=0) == SHAPE and call(B=-3) == SHAPE and call(v_new=FAKE + 2) == SHAPE
    assert call(B=0) == 0


def test_decode_step_rejects_bad_arguments():
    """adr_decode_step checks the new token's arguments on top of the attention's, before any launch."""
    lib = adr.load_library()
    c = cache()

    def call(**kw):
        a = dict(out=FAKE, q=FAKE, k_new=FAKE, v_new=FAKE, stride=2 * 128, bt=FAKE, seq=FAKE, B=2, Hq=8,
                 max_seq_len=64, part=0)
        a.update(kw)
        return lib.adr_decode_step(a["out"], adr.ADR_BF16, None, a["q"], 8 * 128, a["k_new"], a["v_new"],
                                   a["stride"], ctypes.byref(c), a["bt"], 4, a["seq"], a["B"], a["Hq"], 0.1,
                                   a["max_seq_len"], a["part"], None, 0, 0, None)
    assert call(k_new=None) == NULL and call(v_new=None) == NULL
    assert call(out=None) == NULL and call(seq=None) == NULL and call(bt=None) == NULL
    assert call(stride=128) == SHAPE and call(stride=2 * 128 + 4) == SHAPE and call(k_new=FAKE + 2) == SHAPE
    assert call(Hq=7) == SHAPE and call(max_seq_len=65) == SHAPE
    assert call(part=16) == WORK
    assert call(B=0) == 0


def test_merge_rejects_bad_arguments():
    lib = adr.load_library()

    def call(**kw):
        a = dict(out=FAKE, dt=adr.ADR_F32, lse=None, po=FAKE, pl=FAKE, off=FAKE, B=1, heads=4, d=128)
        a.update(kw)
        return lib.adr_lse_merge(a["out"], a["dt"], a["lse"], a["po"], a["pl"], a["off"], a["B"],
                                 a["heads"], a["d"], None)
    assert call(out=None) == NULL and call(po=None) == NULL and call(off=None) == NULL
    assert call(heads=0) == SHAPE and call(d=100) == UNSUP and call(dt=adr.ADR_FP8_E4M3) == UNSUP
    assert call(B=0) == 0


def test_workspace_size_formula():
    control = 256 * 2                            # a status block and one launch block (up to 512 rows)
    assert adr.adr_decode_workspace_bytes(4, 8, 128, 1000, 0) == control      # an unsplit pass: control area only
    rows = 4 * 2 * 8                             # ceil(1000/512) = 2 partitions
    assert adr.adr_decode_workspace_bytes(4, 8, 128, 1000, 512) == rows * 128 * 4 + 256 + control
    assert adr.adr_decode_workspace_bytes(4, 8, 128, 1024, 512) == rows * 128 * 4 + 256 + control
    assert adr.adr_decode_workspace_bytes(4, 8, 128, 1025, 512) > rows * 128 * 4 + 256 + control
    assert adr.adr_decode_workspace_bytes(513, 8, 128, 1000, 0) == 256 * 3    # two launches of the resident kernel
    assert adr.adr_decode_workspace_bytes(0, 8, 128, 1000, 512) == 0
    assert adr.adr_decode_workspace_bytes(4, 8, 128, 1000, -16) == 0


def test_new_flags_are_accepted_and_status_readers_check_their_arguments():
    lib = adr.load_library()
    ok_flags = adr.WORKSPACE_READY | adr.DEBUG_EXPIRE_WAITS | adr.GRID_CUS(64) | adr.SINGLE_PARTITION_ITEMS
    assert attention(cache(), B=0, flags=ok_flags) == 0
    n = ctypes.c_uint32(7)
    assert lib.adr_decode_read_status(None, 1 << 20, 2, 8, 128, 64, 16, ctypes.byref(n)) == NULL
    assert lib.adr_decode_read_status(FAKE, 1 << 20, 2, 8, 128, 64, 16, None) == NULL
    assert lib.adr_decode_read_status(FAKE, 16, 2, 8, 128, 64, 16, ctypes.byref(n)) == WORK      # too small
    assert lib.adr_decode_read_status(FAKE + 16, 1 << 20, 2, 8, 128, 64, 16, ctypes.byref(n)) == WORK  # misaligned
    assert lib.adr_decode_read_status(FAKE, 1 << 20, 0, 8, 128, 64, 16, ctypes.byref(n)) == WORK # no such workspace
    assert n.value == 7
    rec = binding._CBoundsRecord()
    assert lib.adr_debug_bounds_status(ctypes.byref(rec), 0) == UNSUP       # the release build records nothing


def test_kernel_choice_is_reported_by_the_library():
    lib = adr.load_library()
    def choice(c, **kw):
        a = dict(B=256, Hq=32, max_seq_len=8192, part=512, flags=0)
        a.update(kw)
        return lib.adr_decode_kernel_choice(ctypes.byref(c), a["B"], a["Hq"], a["max_seq_len"], a["part"], a["flags"])
    gqa = cache(Hkv=8)
    assert choice(gqa) == adr.KERNEL_MFMA                         # split pass, groups of four: resident kernel
    assert choice(gqa, part=0) == adr.KERNEL_MFMA_GRID            # whole rows: one workgroup per item
    assert choice(gqa, B=128, Hq=64) == adr.KERNEL_MFMA_GRID      # a small pass of wide groups
    assert choice(gqa, Hq=64) == adr.KERNEL_MFMA                  # 2048 (request, kv-head) pairs
    assert choice(cache(Hkv=8, d=64)) == adr.KERNEL_VALU
    fp8 = cache(Hkv=8, dtype=adr.ADR_FP8_E4M3, k_scale=FAKE, v_scale=FAKE)
    assert choice(fp8) == adr.KERNEL_MFMA and choice(fp8, part=0) == adr.KERNEL_MFMA
    assert choice(gqa, flags=adr.KERNEL_VALU) == adr.KERNEL_VALU
    assert choice(gqa, Hq=128, flags=adr.KERNEL_VALU) == -UNSUP   # groups of sixteen
    assert choice(gqa, Hq=7) == -SHAPE and choice(cache(d=96)) == -UNSUP
    assert lib.adr_kernel_name(adr.KERNEL_MFMA) == b"decode_stream_kernel"
    assert lib.adr_kernel_name(adr.KERNEL_MFMA_GRID) == b"decode_mfma_kernel"
    assert lib.adr_kernel_name(adr.KERNEL_VALU) == b"decode_valu_kernel"
    assert lib.adr_kernel_name(0) == b""


def test_cu_mask_stream_and_fault_count_reject_bad_arguments():
    lib = adr.load_library()
    handle = ctypes.c_void_p()
    one = (ctypes.c_uint32 * 1)(1)
    zero = (ctypes.c_uint32 * 2)(0, 0)
    assert lib.adr_stream_create_cu_mask(None, one, 1) == NULL
    assert lib.adr_stream_create_cu_mask(ctypes.byref(handle), None, 1) == NULL
    assert lib.adr_stream_create_cu_mask(ctypes.byref(handle), one, 0) == SHAPE
    assert lib.adr_stream_create_cu_mask(ctypes.byref(handle), zero, 2) == SHAPE
    assert handle.value is None
    assert lib.adr_stream_destroy(None) == NULL
    assert lib.adr_stream_fault_count(None) == NULL


def test_glue_copies_reject_bad_arguments():
    lib = adr.load_library()
    def pack(**kw):
        a = dict(dst=FAKE, ds=6 * 128, q=FAKE, qs=4 * 128, k=FAKE, ks=128, v=FAKE, vs=128, B=3, Hq=4, Hkv=1, d=128)
        a.update(kw)
        return lib.adr_pack_qkv(a["dst"], a["ds"], a["q"], a["qs"], a["k"], a["ks"], a["v"], a["vs"], a["B"],
                                a["Hq"], a["Hkv"], a["d"], None)
    assert pack(dst=None) == NULL and pack(v=None) == NULL
    assert pack(d=100) == SHAPE and pack(ds=6 * 128 - 8) == SHAPE and pack(qs=4 * 128 + 4) == SHAPE
    assert pack(q=FAKE + 8) == SHAPE and pack(B=-1) == SHAPE
    assert pack(B=0) == 0
    def scatter(**kw):
        a = dict(dst=FAKE, ds=256, rows=8, src=FAKE, ss=256, idx=FAKE, n=4, elems=256)
        a.update(kw)
        return lib.adr_scatter_rows(a["dst"], a["ds"], a["rows"], a["src"], a["ss"], a["idx"], a["n"], a["elems"], None)
    assert scatter(idx=None) == NULL and scatter(src=None) == NULL
    assert scatter(elems=100) == SHAPE and scatter(ds=128) == SHAPE and scatter(ss=260) == SHAPE
    assert scatter(n=0) == 0


def test_graph_table_rejects_bad_arguments_before_recording():
    lib = adr.load_library()
    handle = ctypes.c_void_p()
    caches = (binding._CCache * 1)(cache())
    desc = binding._CStepBuffers(FAKE, adr.ADR_BF16, None, FAKE, 8 * 128, FAKE, FAKE, 2 * 128, caches, 1, FAKE, 4, FAKE, 8,
                                 0.1, 64, 0, None, 0, 0)
    assert lib.adr_graph_table_create(None, ctypes.byref(desc), 4, 8, FAKE) == NULL
    assert lib.adr_graph_table_create(ctypes.byref(handle), None, 4, 8, FAKE) == NULL
    assert lib.adr_graph_table_create(ctypes.byref(handle), ctypes.byref(desc), 4, 8, None) == NULL   # needs a stream to record from
    assert lib.adr_graph_table_create(ctypes.byref(handle), ctypes.byref(desc), 0, 8, FAKE) == SHAPE
    assert lib.adr_graph_table_create(ctypes.byref(handle), ctypes.byref(desc), 3, 8, FAKE) == SHAPE   # 8 is not a multiple of 3
    assert lib.adr_graph_table_create(ctypes.byref(handle), ctypes.byref(desc), 8, 4, FAKE) == SHAPE
    desc.n_layers = 0
    assert lib.adr_graph_table_create(ctypes.byref(handle), ctypes.byref(desc), 4, 8, FAKE) == SHAPE
    assert handle.value is None
    assert lib.adr_graph_table_launch(None, 1, None) == NULL and lib.adr_graph_table_destroy(None) == NULL
    assert lib.adr_graph_table_capacity(None, 1) == -1
