"""GPU parity with cache pages of 32 and 64 tokens (the kernels work in 16-token tiles; a page is
two or four consecutive tiles of the pool): adr_decode_step against the fp64 oracle's append and
attention on the same bytes, pools compared bit for bit."""
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

# lengths after the append: around tile, page and partition boundaries, one padded row
LENS = [1, 16, 17, 31, 32, 33, 63, 64, 65, 0, 96, 97, 127, 128, 129, 511, 512, 513, 1000, 1025, 2100]


def make_case(seed, Hq, Hkv, d, page_size, lens_after):
    lens_after = np.asarray(lens_after, dtype=np.int32)
    wl = W.Workload(97, "pages", B=len(lens_after), Hq=Hq, Hkv=Hkv, d=d, lengths="given", page_size=page_size)
    mb = W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=seed,
                      lens_before=np.maximum(lens_after - 1, 0))
    return wl, types.SimpleNamespace(block_table=mb.block_table, num_pages=mb.num_pages, used=mb.used, q=mb.q,
                                     k_new=mb.k_new, v_new=mb.v_new, k_cache=mb.k_cache, v_cache=mb.v_cache,
                                     seq_lens=lens_after.copy(), positions=(lens_after - 1).astype(np.int32))


@pytest.mark.parametrize("page_size", [32, 64])
@pytest.mark.parametrize("kernel", ["valu", "mfma", "grid", "auto"])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 128), (32, 8, 128), (8, 8, 64)])
@pytest.mark.parametrize("partition_tokens", [0, 64, 512])
def test_bf16_step_matches_oracle(page_size, kernel, Hq, Hkv, d, partition_tokens):
    if d == 64 and kernel in ("mfma", "grid"):
        pytest.skip("the matrix-core kernels serve d = 128")
    wl, b = make_case(3 + page_size + Hq, Hq, Hkv, d, page_size, LENS)
    say("page %d %s Hq=%d Hkv=%d d=%d part=%d" % (page_size, kernel, Hq, Hkv, d, partition_tokens))
    kc, vc = dev(b.k_cache), dev(b.v_cache)
    out = torch.full((wl.B, Hq, d), float("nan"), dtype=torch.float32, device="cuda:0")
    lse = torch.full((wl.B, Hq), float("nan"), dtype=torch.float32, device="cuda:0")
    max_len = int(b.seq_lens.max())
    nbytes = adr.adr_decode_workspace_bytes(wl.B, Hq, d, max_len, partition_tokens)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0") if nbytes else None
    adr.adr_decode_step(out, dev(b.q), dev(b.k_new), dev(b.v_new), adr.KVCache(kc, vc), dev(b.block_table),
                        dev(b.seq_lens), wl.scale, max_len, partition_tokens, ws, lse, KERNELS[kernel])
    torch.cuda.synchronize()
    kh, vh = W.bits(b.k_cache).copy(), W.bits(b.v_cache).copy()
    oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, b.positions)
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)
    ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), kh, vh, b.block_table, b.seq_lens, wl.scale)
    max_abs, _ = compare(out, lse, ref, ref_lse, what="page %d %s" % (page_size, kernel))
    assert max_abs <= ATOL


@pytest.mark.parametrize("page_size", [32, 64])
@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_fp8_step_is_byte_exact_and_matches_oracle(page_size, kernel):
    Hq, Hkv, d = 32, 8, 128
    wl, b = make_case(41 + page_size, Hq, Hkv, d, page_size, LENS)
    say("page %d fp8 %s" % (page_size, kernel))
    k8, ks = W.quantize_pool_fp8(dev(b.k_cache), b.used)
    v8, vs = W.quantize_pool_fp8(dev(b.v_cache), b.used)
    kh, vh, ksh, vsh = (W.bits(t).copy() for t in (k8, v8, ks, vs))
    oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, b.positions, k_scale=ksh, v_scale=vsh)
    out = torch.full((wl.B, Hq, d), float("nan"), dtype=torch.float32, device="cuda:0")
    lse = torch.full((wl.B, Hq), float("nan"), dtype=torch.float32, device="cuda:0")
    max_len = int(b.seq_lens.max())
    ws = torch.empty(adr.adr_decode_workspace_bytes(wl.B, Hq, d, max_len, 512), dtype=torch.uint8, device="cuda:0")
    adr.adr_decode_step(out, dev(b.q), dev(b.k_new), dev(b.v_new), adr.KVCache(k8, v8, ks, vs), dev(b.block_table),
                        dev(b.seq_lens), wl.scale, max_len, 512, ws, lse, KERNELS[kernel])
    torch.cuda.synchronize()
    assert np.array_equal(W.bits(k8), kh) and np.array_equal(W.bits(v8), vh)
    assert np.array_equal(W.bits(ks).view(np.uint32), ksh.view(np.uint32))
    assert np.array_equal(W.bits(vs).view(np.uint32), vsh.view(np.uint32))
    ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), kh, vh, b.block_table, b.seq_lens, wl.scale,
                                              k_scale=ksh, v_scale=vsh)
    compare(out, lse, ref, ref_lse, what="page %d fp8 %s" % (page_size, kernel))
