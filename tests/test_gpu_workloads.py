"""GPU parity at the benchmark's full sizes, in the launch configuration the
benchmark times (same partition size, automatic kernel choice, bf16 output),
against the fp64 oracle: every row of every workload, every resident layer of
the benchmark workload."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_20552_amd as adr
import workloads as W
from gpu_util import ATOL, compare, dev, gpu_attention, oracle_attention, say

pytestmark = pytest.mark.gpu


def run_workload(ident, rows=None, flags=adr.KERNEL_AUTO):
    wl = W.WORKLOADS[ident]
    b = W.make_batch(wl, device="cuda:0")
    info = W.describe_lengths(b.seq_lens)
    say("workload %d %s lengths %s pages %d" % (ident, wl.name, info, b.num_pages))
    cache = adr.KVCache(b.k_cache, b.v_cache)
    table, pos, seq = dev(b.block_table), dev(b.positions), dev(b.seq_lens)
    k0, v0 = b.k_cache.clone(), b.v_cache.clone()
    adr.adr_kv_append(cache, b.k_new, b.v_new, table, pos)
    torch.cuda.synchronize()
    # append: exactly the named slots changed, to exactly the new bits
    pages = torch.from_numpy(b.block_table[np.arange(wl.B), b.positions // 16].astype(np.int64)).cuda()
    slots = torch.from_numpy((b.positions % 16).astype(np.int64)).cuda()
    assert torch.equal(b.k_cache[pages, slots].view(torch.int16), b.k_new.view(torch.int16))
    assert torch.equal(b.v_cache[pages, slots].view(torch.int16), b.v_new.view(torch.int16))
    k0[pages, slots] = b.k_new; v0[pages, slots] = b.v_new
    assert torch.equal(k0.view(torch.int16), b.k_cache.view(torch.int16))
    assert torch.equal(v0.view(torch.int16), b.v_cache.view(torch.int16))
    del k0, v0

    max_len = int(b.seq_lens.max())
    res = {}
    for dt in (torch.bfloat16, torch.float32):
        out, lse = gpu_attention(b.q, b.k_cache, b.v_cache, table, seq, wl.scale,
                                 partition_tokens=wl.partition_tokens, flags=flags, out_dtype=dt,
                                 max_seq_len=max_len)
        res[dt] = (out, lse)
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, wl.scale, rows=rows)
    for dt, (out, lse) in res.items():
        max_abs, max_rel = compare(out, lse, ref, ref_lse, rows=rows, what="workload %d %s" % (ident, dt))
        say("workload %d out=%s max_abs %.3e max_rel %.3e" % (ident, dt, max_abs, max_rel))
        if dt == torch.float32:
            assert max_abs <= ATOL


def test_workload_2_llama2_7b_mha_all_rows():
    run_workload(2)


def test_workload_3_llama3_8b_gqa_one_layer_all_rows():
    run_workload(3)


@pytest.mark.parametrize("layer", range(1, 32))
def test_workload_3_other_resident_layers_all_rows(layer):
    """The benchmark rotates over 32 layer caches; each of layers 1..31 (its own pool values, the same
    page table) is checked like layer 0, after the step's append."""
    wl = W.WORKLOADS[3]
    b = W.make_batch(wl, device="cuda:0")
    kc, vc = W.layer_pools(wl, b, layer, "cuda:0")
    b.k_cache = b.v_cache = None
    table, pos, seq = dev(b.block_table), dev(b.positions), dev(b.seq_lens)
    say("workload 3 layer %d" % layer)
    adr.adr_kv_append(adr.KVCache(kc, vc), b.k_new, b.v_new, table, pos)
    out, lse = gpu_attention(b.q, kc, vc, table, seq, wl.scale, partition_tokens=wl.partition_tokens,
                             out_dtype=torch.bfloat16, max_seq_len=int(b.seq_lens.max()))
    ref, ref_lse = oracle_attention(b.q, kc, vc, b.block_table, b.seq_lens, wl.scale)
    compare(out, lse, ref, ref_lse, what="workload 3 layer %d" % layer)


def test_workload_4_colocation_shape_all_rows():
    run_workload(4)


def test_workload_5_length_skew_all_rows():
    """All 512 rows, the 51 long ones included: the shape whose items are runs of four partitions."""
    run_workload(5)


def test_workload_5_fp8_cache_append_then_attend_all_rows():
    """The fp8 leg of the skew workload at full size: the pools are quantised with library casts,
    the step's token is appended by the fp8 append kernel (bytes and scales checked against the
    oracle's rule on the touched pages), then attention runs as the benchmark runs it and every
    row is compared with the oracle on the dequantised values."""
    wl = W.WORKLOADS[5]
    b = W.make_batch(wl, device="cuda:0")
    k8, ks = W.quantize_pool_fp8(b.k_cache, b.used)
    v8, vs = W.quantize_pool_fp8(b.v_cache, b.used)
    b.k_cache = b.v_cache = None
    torch.cuda.empty_cache()
    rows = np.arange(wl.B, dtype=np.int32)
    say("workload 5 fp8: all %d rows, %d pages" % (len(rows), b.num_pages))
    table, pos, seq = dev(b.block_table), dev(b.positions), dev(b.seq_lens)
    # host copies of the pages the sampled rows' appends touch, before the append
    pages = b.block_table[rows, b.positions[rows] // 16]
    before = [t[torch.from_numpy(pages.astype(np.int64)).cuda()].cpu().numpy() for t in (k8, v8, ks, vs)]
    adr.adr_kv_append(adr.KVCache(k8, v8, ks, vs), b.k_new, b.v_new, table, pos)
    torch.cuda.synchronize()
    # the oracle's append on a miniature pool made of just those pages
    mini_table = np.arange(len(rows), dtype=np.int32)[:, None]
    kh, vh, ksh, vsh = (a.copy() for a in before)
    oracle.kv_append(kh, vh, W.bits(b.k_new)[rows], W.bits(b.v_new)[rows], mini_table,
                     (b.positions[rows] % 16).astype(np.int32), k_scale=ksh, v_scale=vsh)
    after = [t[torch.from_numpy(pages.astype(np.int64)).cuda()].cpu().numpy() for t in (k8, v8, ks, vs)]
    assert np.array_equal(after[0], kh) and np.array_equal(after[1], vh)
    assert np.array_equal(after[2].view(np.uint32), ksh.view(np.uint32))
    assert np.array_equal(after[3].view(np.uint32), vsh.view(np.uint32))

    out, lse = gpu_attention(b.q, k8, v8, table, seq, wl.scale, partition_tokens=wl.partition_tokens,
                             out_dtype=torch.float32, max_seq_len=int(b.seq_lens.max()), k_scale=ks, v_scale=vs)
    ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), W.bits(k8), W.bits(v8), b.block_table, b.seq_lens,
                                              wl.scale, k_scale=W.bits(ks), v_scale=W.bits(vs))
    max_abs, max_rel = compare(out, lse, ref, ref_lse, what="workload 5 fp8")
    say("workload 5 fp8 max_abs %.3e max_rel %.3e" % (max_abs, max_rel))
    assert max_abs <= ATOL


def test_resident_kernel_reports_no_expired_waits():
    """Runs after the cases above: none of the waves' bounded waits may have expired."""
    assert adr.adr_stream_fault_count() == 0
