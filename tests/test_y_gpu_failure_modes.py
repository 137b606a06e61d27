"""What the resident kernel does when a hand-shake between its waves breaks.  The condition is forced
from the host (ADR_DEBUG_EXPIRE_WAITS makes every wait on another wave give up at once); every kernel
still runs to its end.  No row may then pass as a result: out and lse come back as NaN, the expiry is
counted in the workspace's status block and device-wide, and the next ordinary call on the same
buffers is clean.  (This file sorts behind the tests that require the device-wide count to be zero.)"""
import numpy as np
import pytest
import torch

import paper_2503_20552_amd as adr
import workloads as W
from gpu_util import compare, dev, oracle_attention, say

pytestmark = pytest.mark.gpu


def case(seed, lens, Hq=32, Hkv=8):
    wl = W.Workload(96, "case", B=len(lens), Hq=Hq, Hkv=Hkv, d=128, lengths="given")
    return W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=seed,
                        lens_before=np.asarray(lens, dtype=np.int32))


def buffers(b, out_dtype):
    wl = b.wl
    out = torch.zeros((wl.B, wl.Hq, wl.d), dtype=out_dtype, device="cuda:0")
    lse = torch.zeros((wl.B, wl.Hq), dtype=torch.float32, device="cuda:0")
    return out, lse


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("partition_tokens", [0, 64, 512])
@pytest.mark.parametrize("fp8", [False, True])
def test_expired_waits_turn_the_call_into_nan_and_are_counted(out_dtype, partition_tokens, fp8):
    b = case(71, [700, 1, 64, 65, 513, 2000, 0, 31])
    max_len = int(b.seq_lens.max())
    wl = b.wl
    if fp8:
        k, ks = W.quantize_pool_fp8(dev(b.k_cache), b.used)
        v, vs = W.quantize_pool_fp8(dev(b.v_cache), b.used)
        cache = adr.KVCache(k, v, ks, vs)
    else:
        cache = adr.KVCache(dev(b.k_cache), dev(b.v_cache))
    q, table, seq = dev(b.q), dev(b.block_table), dev(b.seq_lens)
    n = adr.adr_decode_workspace_bytes(wl.B, wl.Hq, wl.d, max_len, partition_tokens)
    ws = torch.zeros(n // 4, dtype=torch.float32, device="cuda:0")
    out, lse = buffers(b, out_dtype)
    faults_before = adr.adr_stream_fault_count()
    say("forced expiry, partition %d, out %s, fp8 %s" % (partition_tokens, out_dtype, fp8))
    adr.adr_decode_attention(out, q, cache, table, seq, wl.scale, max_len, partition_tokens, ws, lse,
                             adr.KERNEL_MFMA | adr.DEBUG_EXPIRE_WAITS)
    torch.cuda.synchronize()
    assert torch.isnan(out.float()).all(), "a row passed as a result after a wait expired"
    assert torch.isnan(lse).all()
    assert adr.adr_decode_read_status(ws, wl.B, wl.Hq, wl.d, max_len, partition_tokens) > 0
    assert adr.adr_stream_fault_count() > faults_before
    # the same buffers, an ordinary call: clean, and the status block starts from zero again
    adr.adr_decode_attention(out, q, cache, table, seq, wl.scale, max_len, partition_tokens, ws, lse, adr.KERNEL_MFMA)
    torch.cuda.synchronize()
    if fp8:
        import oracle
        ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), W.bits(cache.k), W.bits(cache.v), b.block_table,
                                                  b.seq_lens, wl.scale, k_scale=W.bits(cache.k_scale),
                                                  v_scale=W.bits(cache.v_scale))
    else:
        ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, wl.scale)
    compare(out, lse, ref, ref_lse, what="after the forced failure")
    assert adr.adr_decode_read_status(ws, wl.B, wl.Hq, wl.d, max_len, partition_tokens) == 0


def test_expired_waits_without_a_workspace_poison_the_rows_too():
    b = case(72, [300, 1, 17, 900])
    wl = b.wl
    max_len = int(b.seq_lens.max())
    cache = adr.KVCache(dev(b.k_cache), dev(b.v_cache))
    q, table, seq = dev(b.q), dev(b.block_table), dev(b.seq_lens)
    out, lse = buffers(b, torch.float32)
    say("forced expiry, no workspace")
    adr.adr_decode_attention(out, q, cache, table, seq, wl.scale, max_len, 0, None, lse,
                             adr.KERNEL_MFMA | adr.DEBUG_EXPIRE_WAITS)
    torch.cuda.synchronize()
    assert torch.isnan(out).all() and torch.isnan(lse).all()
    adr.adr_decode_attention(out, q, cache, table, seq, wl.scale, max_len, 0, None, lse, adr.KERNEL_MFMA)
    torch.cuda.synchronize()
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, wl.scale)
    compare(out, lse, ref, ref_lse, what="after the forced failure, no workspace")


def test_partials_of_a_failed_pass_make_the_later_merge_return_nan():
    b = case(73, [700, 64, 65, 2000])
    wl = b.wl
    max_len = int(b.seq_lens.max())
    cache = adr.KVCache(dev(b.k_cache), dev(b.v_cache))
    q, table, seq = dev(b.q), dev(b.block_table), dev(b.seq_lens)
    n = adr.adr_decode_workspace_bytes(wl.B, wl.Hq, wl.d, max_len, 512)
    ws = torch.zeros(n // 4, dtype=torch.float32, device="cuda:0")
    out, lse = buffers(b, torch.float32)
    say("forced expiry, partials only, then merge")
    adr.adr_decode_attention(out, q, cache, table, seq, wl.scale, max_len, 512, ws, lse,
                             adr.KERNEL_MFMA | adr.DEBUG_EXPIRE_WAITS | adr.PARTIALS_ONLY)
    out.zero_(); lse.zero_()
    adr.adr_decode_merge(out, seq, max_len, 512, ws, lse)
    torch.cuda.synchronize()
    assert torch.isnan(out).all() and torch.isnan(lse).all()
