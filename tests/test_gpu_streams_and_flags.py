"""GPU tests of what surrounds the kernels' arithmetic: many attention launches queued on two streams at
once (each call's counters live in its own workspace), the flag that vouches for a cleared control area,
the flag that sizes the resident kernel's grid, and the debug build's record of out-of-range table
entries.  Every result is compared with the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_20552_amd as adr
import workloads as W
from gpu_util import compare, dev, gpu_attention, oracle_attention, say

pytestmark = pytest.mark.gpu


def small_case(seed, Hq, Hkv, d, lens, pool_pages=0):
    wl = W.Workload(97, "case", B=len(lens), Hq=Hq, Hkv=Hkv, d=d, lengths="given", fixed_pool_pages=pool_pages)
    return W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=seed,
                        lens_before=np.asarray(lens, dtype=np.int32))


class Resident:
    """One case's tensors on the device."""
    def __init__(self, b):
        self.b = b
        self.q, self.kc, self.vc = dev(b.q), dev(b.k_cache), dev(b.v_cache)
        self.table, self.seq = dev(b.block_table), dev(b.seq_lens)
        self.cache = adr.KVCache(self.kc, self.vc)
        self.max_len = int(b.seq_lens.max())
        wl = b.wl
        self.shape = (wl.B, wl.Hq, wl.d)

    def workspace(self, partition_tokens):
        n = adr.adr_decode_workspace_bytes(*self.shape, self.max_len, partition_tokens)
        return torch.full((n // 4,), float("nan"), dtype=torch.float32, device="cuda:0")


def test_two_streams_with_more_than_128_queued_launches_each():
    """160 split and 160 unsplit launches of the resident kernel per stream, queued without a wait in
    between, the two streams running side by side.  Every launch has a workspace of its own (the unsplit
    ones the small control-only one), so no two launches that can overlap share counters."""
    rng = np.random.default_rng(11)
    cases = [Resident(small_case(61, 32, 8, 128, rng.integers(1, 700, size=12))),
             Resident(small_case(62, 16, 4, 128, rng.integers(1, 500, size=9)))]
    refs = [oracle_attention(c.b.q, c.b.k_cache, c.b.v_cache, c.b.block_table, c.b.seq_lens, c.b.wl.scale)
            for c in cases]
    n = 160
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]            # default priority
    outs, lses, spaces = [], [], []
    for c in cases:
        outs.append(torch.full((2 * n,) + c.shape, float("nan"), dtype=torch.float32, device="cuda:0"))
        lses.append(torch.full((2 * n,) + c.shape[:2], float("nan"), dtype=torch.float32, device="cuda:0"))
        spaces.append([c.workspace(64) for _ in range(n)] + [c.workspace(0) for _ in range(n)])
    torch.cuda.synchronize()
    say("two streams x %d queued attention launches" % (2 * n))
    for i in range(2 * n):
        for c, stream, out, lse, ws in zip(cases, streams, outs, lses, spaces):
            part = 64 if i < n else 0
            adr.adr_decode_attention(out[i], c.q, c.cache, c.table, c.seq, c.b.wl.scale, c.max_len, part, ws[i],
                                     lse[i], adr.KERNEL_MFMA, stream=stream)
    torch.cuda.synchronize()
    for c, out, lse, ws, (ref, ref_lse) in zip(cases, outs, lses, spaces, refs):
        # identical launches give identical bits; one of each kind is compared with the oracle
        assert torch.equal(out[:n], out[0].expand_as(out[:n])) and torch.equal(out[n:], out[n].expand_as(out[n:]))
        assert torch.equal(lse[:n], lse[0].expand_as(lse[:n])) and torch.equal(lse[n:], lse[n].expand_as(lse[n:]))
        compare(out[0], lse[0], ref, ref_lse, what="split launch")
        compare(out[n], lse[n], ref, ref_lse, what="unsplit launch")
        assert adr.adr_decode_read_status(ws[0], *c.shape, c.max_len, 64) == 0
        assert adr.adr_decode_read_status(ws[n], *c.shape, c.max_len, 0) == 0


def test_workspace_ready_flag_skips_the_clearing_kernel_and_changes_nothing():
    c = Resident(small_case(63, 32, 8, 128, [700, 1, 64, 65, 513, 2000]))
    ref, ref_lse = oracle_attention(c.b.q, c.b.k_cache, c.b.v_cache, c.b.block_table, c.b.seq_lens, c.b.wl.scale)
    ws = c.workspace(512)
    out = [torch.full(c.shape, float("nan"), dtype=torch.float32, device="cuda:0") for _ in range(3)]
    lse = [torch.full(c.shape[:2], float("nan"), dtype=torch.float32, device="cuda:0") for _ in range(3)]
    say("ADR_WORKSPACE_READY")
    adr.adr_decode_attention(out[0], c.q, c.cache, c.table, c.seq, c.b.wl.scale, c.max_len, 512, ws, lse[0],
                             adr.KERNEL_MFMA)
    for i in (1, 2):    # the first call left the control area cleared, and so does every later one
        adr.adr_decode_attention(out[i], c.q, c.cache, c.table, c.seq, c.b.wl.scale, c.max_len, 512, ws, lse[i],
                                 adr.KERNEL_MFMA | adr.WORKSPACE_READY)
    torch.cuda.synchronize()
    compare(out[0], lse[0], ref, ref_lse, what="cleared by the call")
    assert torch.equal(out[0], out[1]) and torch.equal(out[0], out[2])
    assert torch.equal(lse[0], lse[1]) and torch.equal(lse[0], lse[2])
    assert adr.adr_decode_read_status(ws, *c.shape, c.max_len, 512) == 0


@pytest.mark.parametrize("cus", [1, 7, 64, 4095])
def test_grid_sized_by_flag_gives_the_same_results(cus):
    rng = np.random.default_rng(5)
    c = Resident(small_case(64, 32, 8, 128, rng.integers(1, 1500, size=40)))
    ref, ref_lse = oracle_attention(c.b.q, c.b.k_cache, c.b.v_cache, c.b.block_table, c.b.seq_lens, c.b.wl.scale)
    say("ADR_GRID_CUS(%d)" % cus)
    out, lse = gpu_attention(c.q, c.kc, c.vc, c.table, c.seq, c.b.wl.scale, partition_tokens=512,
                             flags=adr.KERNEL_MFMA | adr.GRID_CUS(cus))
    compare(out, lse, ref, ref_lse, what="grid for %d units" % cus)
    base, base_lse = gpu_attention(c.q, c.kc, c.vc, c.table, c.seq, c.b.wl.scale, partition_tokens=512,
                                   flags=adr.KERNEL_MFMA)
    assert torch.equal(out, base) and torch.equal(lse, base_lse)   # the result does not depend on the grid


@pytest.mark.parametrize("kernel", [adr.KERNEL_MFMA, adr.KERNEL_MFMA_GRID, adr.KERNEL_VALU])
def test_debug_build_records_out_of_range_entries_and_computes_what_the_release_build_computes(kernel):
    b = small_case(65, 8, 2, 128, [40, 40, 200])
    table = b.block_table.copy()
    table[1, 0] = -5                               # clamps to page 0
    table[2, 3] = b.num_pages + 1000               # clamps to the last page
    kc = torch.nan_to_num(b.k_cache.float(), nan=0.5).to(torch.bfloat16)      # the clamped pages are read
    vc = torch.nan_to_num(b.v_cache.float(), nan=0.5).to(torch.bfloat16)
    args = (dev(b.q), dev(kc), dev(vc), dev(table), dev(b.seq_lens), b.wl.scale)
    say("debug build, kernel %d" % kernel)
    release, release_lse = gpu_attention(*args, partition_tokens=64, flags=kernel)
    with adr.debug_library():
        adr.adr_debug_bounds_status(reset=True)
        debug, debug_lse = gpu_attention(*args, partition_tokens=64, flags=kernel)
        rec = adr.adr_debug_bounds_status(reset=True)
        assert rec["kind"] == 1 and rec["count"] >= 2
        assert (rec["row"], rec["index"], rec["value"]) in ((1, 0, -5), (2, 3, b.num_pages + 1000))
        # a clean table leaves the record empty
        clean = np.clip(table, 0, b.num_pages - 1).astype(np.int32)
        again, _ = gpu_attention(args[0], args[1], args[2], dev(clean), args[4], args[5], partition_tokens=64,
                                 flags=kernel)
        assert adr.adr_debug_bounds_status()["count"] == 0
        # append: a position past the row's table, then a page id outside the pool
        pos = b.positions.copy()
        pos[0] = b.block_table.shape[1] * 16 + 3       # past the table
        pos[1] = 5                                     # table[1, 0] is not a page of the pool
        cache = adr.KVCache(dev(kc), dev(vc))
        before = cache.k.clone()
        adr.adr_kv_append(cache, dev(b.k_new), dev(b.v_new), dev(table), dev(pos))
        torch.cuda.synchronize()
        rec = adr.adr_debug_bounds_status(reset=True)
        assert rec["count"] == 2 and rec["kind"] in (2, 3)
        assert torch.equal(cache.k[table[0, 0]], before[table[0, 0]])         # the skipped row wrote nothing
    assert torch.equal(release, debug) and torch.equal(release_lse, debug_lse) and torch.equal(release, again)
    with pytest.raises(adr.AdrError):
        adr.adr_debug_bounds_status()                  # the release build has no such record


@pytest.mark.parametrize("Hq,Hkv", [(64, 8), (32, 8)])
def test_many_one_page_rows_launched_back_to_back(Hq, Hkv):
    """128 rows of one page each (every item is a single page, three waves of four have nothing to do and the
    workgroups spend their time handing out and finishing items), sixty launches in a row on one cleared
    workspace: the regime where the hand-over between items is all there is."""
    b = small_case(66, Hq, Hkv, 128, np.full(128, 15))
    c = Resident(b)
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.wl.scale)
    ws = c.workspace(512)
    outs = torch.full((60,) + c.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    lses = torch.full((60,) + c.shape[:2], float("nan"), dtype=torch.float32, device="cuda:0")
    say("one-page rows, 60 launches, Hq=%d" % Hq)
    for i in range(60):
        adr.adr_decode_attention(outs[i], c.q, c.cache, c.table, c.seq, b.wl.scale, c.max_len, 512, ws, lses[i],
                                 adr.KERNEL_MFMA | (adr.WORKSPACE_READY if i else 0))
    torch.cuda.synchronize()
    compare(outs[0], lses[0], ref, ref_lse, what="one-page rows")
    assert torch.equal(outs, outs[0].expand_as(outs)) and torch.equal(lses, lses[0].expand_as(lses))
    assert adr.adr_decode_read_status(ws, *c.shape, c.max_len, 512) == 0
