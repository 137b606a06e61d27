"""adr_decode_attention_static: the entry point for callers that cannot allocate.  Its workspace is a
static device array inside the library; everything else is adr_decode_attention.  Two calls in a row
through the C ABI, the second with a smaller input, each compared bit for bit with adr_decode_attention
on a caller's workspace and, within the floating-point gate, with the fp64 oracle.  Collected last."""
import numpy as np
import pytest
import torch

import paper_2503_20552_amd as adr
import workloads as W
from gpu_util import ATOL, compare, dev, oracle_attention, say

pytestmark = pytest.mark.gpu


def case(seed, lens):
    wl = W.Workload(95, "case", B=len(lens), Hq=32, Hkv=8, d=128, lengths="given")
    return W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=seed,
                        lens_before=np.asarray(lens, dtype=np.int32))


def run_both(b, partition_tokens, flags):
    wl = b.wl
    max_len = int(b.seq_lens.max())
    cache = adr.KVCache(dev(b.k_cache), dev(b.v_cache))
    q, table, seq = dev(b.q), dev(b.block_table), dev(b.seq_lens)
    shape = (wl.B, wl.Hq, wl.d)
    res = []
    for static in (True, False):
        out = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
        lse = torch.full(shape[:2], float("nan"), dtype=torch.float32, device="cuda:0")
        if static:
            adr.adr_decode_attention_static(out, q, cache, table, seq, wl.scale, max_len, partition_tokens, lse, flags)
        else:
            n = adr.adr_decode_workspace_bytes(*shape, max_len, partition_tokens)
            ws = torch.full((n // 4,), float("nan"), dtype=torch.float32, device="cuda:0")
            adr.adr_decode_attention(out, q, cache, table, seq, wl.scale, max_len, partition_tokens, ws, lse, flags)
        torch.cuda.synchronize()
        res.append((out, lse))
    return res


@pytest.mark.parametrize("flags", [adr.KERNEL_AUTO, adr.KERNEL_MFMA_GRID, adr.KERNEL_VALU])
def test_static_workspace_entry_matches_the_caller_workspace_entry_twice_in_a_row(flags):
    rng = np.random.default_rng(17)
    first = case(81, np.concatenate([rng.integers(1, 3000, size=22), [0, 2999]]))     # 24 rows, up to 6 partitions
    second = case(82, rng.integers(1, 600, size=5))                                   # smaller in every respect
    for name, b in (("first", first), ("second, smaller", second)):
        say("static workspace entry, %s call, flags %d" % (name, flags))
        (out_s, lse_s), (out_w, lse_w) = run_both(b, 512, flags)
        assert torch.equal(out_s.view(torch.int32), out_w.view(torch.int32)), name
        assert torch.equal(lse_s.view(torch.int32), lse_w.view(torch.int32)), name
        ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.wl.scale)
        max_abs, _ = compare(out_s, lse_s, ref, ref_lse, what="static entry, %s call" % name)
        assert max_abs <= ATOL


def test_static_workspace_entry_serves_unsplit_passes_and_refuses_what_does_not_fit():
    b = case(83, [40, 1, 700])
    say("static workspace entry, unsplit pass and size limit")
    (out_s, lse_s), (out_w, lse_w) = run_both(b, 0, adr.KERNEL_MFMA)
    assert torch.equal(out_s.view(torch.int32), out_w.view(torch.int32))
    assert torch.equal(lse_s.view(torch.int32), lse_w.view(torch.int32))
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.wl.scale)
    compare(out_s, lse_s, ref, ref_lse, what="static entry, unsplit")
    # 3 rows whose table could name 1 M tokens, in partitions of 16: far more partial results than the array holds
    wl = b.wl
    assert adr.adr_decode_workspace_bytes(wl.B, wl.Hq, wl.d, 1 << 20, 16) > adr.STATIC_SCRATCH_BYTES
    wide_table = torch.zeros((wl.B, (1 << 20) // 16), dtype=torch.int32, device="cuda:0")
    out = torch.zeros((wl.B, wl.Hq, wl.d), dtype=torch.float32, device="cuda:0")
    with pytest.raises(adr.AdrError) as err:
        adr.adr_decode_attention_static(out, dev(b.q), adr.KVCache(dev(b.k_cache), dev(b.v_cache)), wide_table,
                                        dev(b.seq_lens), wl.scale, 1 << 20, 16)
    assert err.value.status == 4                                   # ADR_ERR_WORKSPACE, before any launch
    assert torch.all(out == 0)
    with pytest.raises(adr.AdrError) as err:
        adr.adr_decode_attention_static(out, dev(b.q), adr.KVCache(dev(b.k_cache), dev(b.v_cache)),
                                        dev(b.block_table), dev(b.seq_lens), wl.scale, int(b.seq_lens.max()), 512,
                                        None, adr.WORKSPACE_READY)
    assert err.value.status == 3                                   # ADR_ERR_UNSUPPORTED
