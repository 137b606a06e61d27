"""GPU parity of adr_decode_step (append and attention in one call) against the fp64 oracle's
append followed by its attention, and against the library's own two separate calls: the cache
must come out bit-identical to both, the attention output bit-identical to the two-call path
and within the floating-point gate of the oracle."""
import types

import numpy as np
import pytest
import torch

import oracle
import paper_2503_20552_amd as adr
import workloads as W
from gpu_util import ATOL, compare, dev, say

pytestmark = pytest.mark.gpu

KERNELS = {"valu": adr.KERNEL_VALU, "mfma": adr.KERNEL_MFMA, "grid": adr.KERNEL_MFMA_GRID,
           "auto": adr.KERNEL_AUTO}


def make_case(seed, Hq, Hkv, d, lens_after, pool_pages=0):
    """A batch whose rows attend lens_after tokens, the last of which is the step's new one.
    Rows of length 0 are padding: they own no token and nothing is appended for them."""
    lens_after = np.asarray(lens_after, dtype=np.int32)
    before = np.maximum(lens_after - 1, 0)
    wl = W.Workload(98, "step", B=len(lens_after), Hq=Hq, Hkv=Hkv, d=d, lengths="given",
                    fixed_pool_pages=pool_pages)
    mb = W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=seed, lens_before=before)
    b = types.SimpleNamespace(block_table=mb.block_table, num_pages=mb.num_pages, used=mb.used, q=mb.q,
                              k_new=mb.k_new, v_new=mb.v_new, k_cache=mb.k_cache, v_cache=mb.v_cache,
                              seq_lens=lens_after.copy(),
                              positions=(lens_after - 1).astype(np.int32))  # -1 for a padded row
    return wl, b


def run_step(wl, b, flags, partition_tokens, out_dtype=torch.float32, max_seq_len=None, stream=None):
    kc, vc = dev(b.k_cache), dev(b.v_cache)
    q, kn, vn = dev(b.q), dev(b.k_new), dev(b.v_new)
    table, seq = dev(b.block_table), dev(b.seq_lens)
    if max_seq_len is None:
        max_seq_len = int(b.seq_lens.max())
    out = torch.full((wl.B, wl.Hq, wl.d), float("nan"), dtype=out_dtype, device="cuda:0")
    lse = torch.full((wl.B, wl.Hq), float("nan"), dtype=torch.float32, device="cuda:0")
    nbytes = adr.adr_decode_workspace_bytes(wl.B, wl.Hq, wl.d, max_seq_len, partition_tokens)
    ws = torch.full((max(nbytes, 4) // 4,), float("nan"), dtype=torch.float32, device="cuda:0") if nbytes else None
    torch.cuda.synchronize()  # the call may go to another stream than the one that filled the buffers
    adr.adr_decode_step(out, q, kn, vn, adr.KVCache(kc, vc), table, seq, wl.scale, max_seq_len,
                        partition_tokens, ws, lse, flags, stream=stream)
    torch.cuda.synchronize()
    return out, lse, kc, vc


def run_two_calls(wl, b, flags, partition_tokens, out_dtype=torch.float32, max_seq_len=None):
    kc, vc = dev(b.k_cache), dev(b.v_cache)
    q, kn, vn = dev(b.q), dev(b.k_new), dev(b.v_new)
    table, seq = dev(b.block_table), dev(b.seq_lens)
    if max_seq_len is None:
        max_seq_len = int(b.seq_lens.max())
    pos = dev(np.where(b.seq_lens > max_seq_len, -1, b.seq_lens - 1).astype(np.int32))
    out = torch.full((wl.B, wl.Hq, wl.d), float("nan"), dtype=out_dtype, device="cuda:0")
    lse = torch.full((wl.B, wl.Hq), float("nan"), dtype=torch.float32, device="cuda:0")
    nbytes = adr.adr_decode_workspace_bytes(wl.B, wl.Hq, wl.d, max_seq_len, partition_tokens)
    ws = torch.full((max(nbytes, 4) // 4,), float("nan"), dtype=torch.float32, device="cuda:0") if nbytes else None
    cache = adr.KVCache(kc, vc)
    adr.adr_kv_append(cache, kn, vn, table, pos)
    adr.adr_decode_attention(out, q, cache, table, seq, wl.scale, max_seq_len, partition_tokens, ws, lse, flags)
    torch.cuda.synchronize()
    return out, lse, kc, vc


def oracle_step(wl, b, max_seq_len=None):
    kh, vh = W.bits(b.k_cache).copy(), W.bits(b.v_cache).copy()
    lens = b.seq_lens if max_seq_len is None else np.minimum(b.seq_lens, max_seq_len)
    # a row longer than the host's bound is attended up to the bound and appends nothing
    pos = b.seq_lens - 1 if max_seq_len is None else np.where(b.seq_lens > max_seq_len, -1, b.seq_lens - 1)
    oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, pos.astype(np.int32))
    ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), kh, vh, b.block_table, lens.astype(np.int32), wl.scale)
    return ref, ref_lse, kh, vh


# Lengths after the append: single tokens, page and partition boundaries on both sides, a padded
# row, rows of many partitions.
LENS = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 0, 127, 128, 129, 511, 512, 513, 1000, 1024, 1025, 2300, 0, 777]


@pytest.mark.parametrize("kernel", ["mfma", "auto", "grid", "valu"])
@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 2), (32, 8), (16, 1)])
@pytest.mark.parametrize("partition_tokens", [0, 64, 512])
def test_step_equals_append_then_attend(kernel, Hq, Hkv, partition_tokens):
    if kernel == "valu" and Hq // Hkv > 8:
        pytest.skip("the vector-ALU kernel serves groups of up to eight heads")
    wl, b = make_case(7 + Hq + Hkv, Hq, Hkv, 128, LENS)
    say("step %s Hq=%d Hkv=%d part=%d" % (kernel, Hq, Hkv, partition_tokens))
    out, lse, kc, vc = run_step(wl, b, KERNELS[kernel], partition_tokens)
    ref, ref_lse, kh, vh = oracle_step(wl, b)
    # integer part: the whole pool, poison included, bit for bit
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)
    max_abs, _ = compare(out, lse, ref, ref_lse, what="step %s" % kernel)
    assert max_abs <= ATOL
    out2, lse2, kc2, vc2 = run_two_calls(wl, b, KERNELS[kernel], partition_tokens)
    assert torch.equal(kc.view(torch.int16), kc2.view(torch.int16))
    assert torch.equal(vc.view(torch.int16), vc2.view(torch.int16))
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))
    assert torch.equal(lse.view(torch.int32), lse2.view(torch.int32))


def test_step_d64_runs_the_two_kernel_path():
    wl, b = make_case(5, 8, 8, 64, [1, 16, 17, 200, 0, 513])
    say("step d=64")
    out, lse, kc, vc = run_step(wl, b, adr.KERNEL_AUTO, 64)
    ref, ref_lse, kh, vh = oracle_step(wl, b)
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)
    compare(out, lse, ref, ref_lse, what="step d=64")


def test_step_with_a_grouped_qkv_buffer_and_bf16_output():
    """q, k_new and v_new as views into one [B, (Hq+2Hkv) d] buffer, as the executor receives them."""
    Hq, Hkv, d = 32, 8, 128
    wl, b = make_case(11, Hq, Hkv, d, [5, 600, 64, 1, 1500, 0, 48, 49])
    say("step grouped buffer")
    grouped = torch.zeros((wl.B, (Hq + 2 * Hkv) * d), dtype=torch.bfloat16, device="cuda:0")
    adr.adr_pack_qkv(grouped, dev(b.q), dev(b.k_new), dev(b.v_new))
    q = grouped[:, :Hq * d].view(wl.B, Hq, d)
    kn = grouped[:, Hq * d:(Hq + Hkv) * d].view(wl.B, Hkv, d)
    vn = grouped[:, (Hq + Hkv) * d:].view(wl.B, Hkv, d)
    kc, vc = dev(b.k_cache), dev(b.v_cache)
    out = torch.empty((wl.B, Hq, d), dtype=torch.bfloat16, device="cuda:0")
    max_len = int(b.seq_lens.max())
    nbytes = adr.adr_decode_workspace_bytes(wl.B, Hq, d, max_len, 512)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    adr.adr_decode_step(out, q, kn, vn, adr.KVCache(kc, vc), dev(b.block_table), dev(b.seq_lens), wl.scale,
                        max_len, 512, ws, None, adr.KERNEL_MFMA)
    torch.cuda.synchronize()
    ref, ref_lse, kh, vh = oracle_step(wl, b)
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)
    compare(out, None, ref, ref_lse, what="step grouped")


def test_step_skips_rows_whose_last_page_has_no_valid_entry():
    """A table entry outside the pool for the page of the new token: nothing is written for that
    row (as adr_kv_append leaves it), and the row attends what the clamped page holds."""
    wl, b = make_case(13, 8, 2, 128, [40, 100, 33, 700], pool_pages=256)
    say("step invalid page ids")
    bad = b.block_table.copy()
    bad[1, (100 - 1) // 16] = -7
    bad[3, (700 - 1) // 16] = 1 << 20
    b.block_table = bad
    # the clamped pages must hold numbers, not poison, for the attention to be comparable
    for t in (b.k_cache, b.v_cache):
        t[0] = torch.randn(t[0].shape, generator=torch.Generator().manual_seed(1)).to(t.dtype)
        t[-1] = torch.randn(t[-1].shape, generator=torch.Generator().manual_seed(2)).to(t.dtype)
    for kernel in ("mfma", "valu"):
        out, lse, kc, vc = run_step(wl, b, KERNELS[kernel], 64)
        out2, lse2, kc2, vc2 = run_two_calls(wl, b, KERNELS[kernel], 64)
        assert torch.equal(kc.view(torch.int16), kc2.view(torch.int16))
        assert torch.equal(vc.view(torch.int16), vc2.view(torch.int16))
        assert torch.equal(out.view(torch.int32), out2.view(torch.int32))
        # rows 1 and 3 wrote nothing; rows 0 and 2 did
        kh, vh = W.bits(b.k_cache).copy(), W.bits(b.v_cache).copy()
        pos = (b.seq_lens - 1).astype(np.int32)
        pos[[1, 3]] = -1
        oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), np.clip(bad, 0, 255).astype(np.int32), pos)
        assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)


def test_step_row_longer_than_max_seq_len_is_truncated_and_appends_nothing():
    """Rows 0 and 2 exceed the bound: they attend their first 128 tokens and the cache keeps the older
    token that sits at the bound; row 3 is exactly at the bound and appends as usual."""
    wl, b = make_case(17, 8, 2, 128, [300, 50, 129, 128])
    say("step max_seq_len")
    for kernel in ("mfma", "valu"):
        out, lse, kc, vc = run_step(wl, b, KERNELS[kernel], 64, max_seq_len=128)
        ref, ref_lse, kh, vh = oracle_step(wl, b, max_seq_len=128)
        assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)
        before = W.bits(b.k_cache)
        assert np.array_equal(kh[b.block_table[0, 7]], before[b.block_table[0, 7]]), "row 0 must not append"
        compare(out, lse, ref, ref_lse, what="step truncated %s" % kernel)


def test_step_on_a_stream_confined_to_a_few_compute_units():
    """A small grid makes several passes over the rows' copies."""
    wl, b = make_case(19, 32, 8, 128, [int(x) for x in np.random.default_rng(3).integers(1, 900, size=96)])
    say("step on a CU-masked stream")
    handle = adr.adr_stream_create_cu_mask([i < 8 for i in range(torch.cuda.get_device_properties(0).multi_processor_count)])
    try:
        stream = torch.cuda.ExternalStream(handle)
        torch.cuda.synchronize()
        out, lse, kc, vc = run_step(wl, b, adr.KERNEL_MFMA, 512, stream=stream)
    finally:
        torch.cuda.synchronize()
        adr.adr_stream_destroy(handle)
    ref, ref_lse, kh, vh = oracle_step(wl, b)
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)
    compare(out, lse, ref, ref_lse, what="step masked stream")


@pytest.mark.parametrize("kernel", ["mfma", "valu"])
def test_step_fp8_cache_is_byte_exact_then_attends(kernel):
    """An fp8 cache takes the new token through the append kernel inside the same call."""
    wl, b = make_case(23, 32, 8, 128, [1, 16, 17, 33, 0, 600, 512, 1030])
    say("step fp8 %s" % kernel)
    used = b.used
    kc, vc = dev(b.k_cache), dev(b.v_cache)
    k8, ks = W.quantize_pool_fp8(kc, used)
    v8, vs = W.quantize_pool_fp8(vc, used)
    kh, vh, ksh, vsh = (W.bits(t).copy() for t in (k8, v8, ks, vs))
    oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, b.positions, k_scale=ksh, v_scale=vsh)
    out = torch.full((wl.B, wl.Hq, wl.d), float("nan"), dtype=torch.float32, device="cuda:0")
    lse = torch.full((wl.B, wl.Hq), float("nan"), dtype=torch.float32, device="cuda:0")
    max_len = int(b.seq_lens.max())
    ws = torch.empty(adr.adr_decode_workspace_bytes(wl.B, wl.Hq, wl.d, max_len, 512), dtype=torch.uint8, device="cuda:0")
    adr.adr_decode_step(out, dev(b.q), dev(b.k_new), dev(b.v_new), adr.KVCache(k8, v8, ks, vs), dev(b.block_table),
                        dev(b.seq_lens), wl.scale, max_len, 512, ws, lse, KERNELS[kernel])
    torch.cuda.synchronize()
    assert np.array_equal(W.bits(k8), kh) and np.array_equal(W.bits(v8), vh)
    assert np.array_equal(W.bits(ks).view(np.uint32), ksh.view(np.uint32))
    assert np.array_equal(W.bits(vs).view(np.uint32), vsh.view(np.uint32))
    ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), kh, vh, b.block_table, b.seq_lens, wl.scale,
                                              k_scale=ksh, v_scale=vsh)
    compare(out, lse, ref, ref_lse, what="step fp8 %s" % kernel)
