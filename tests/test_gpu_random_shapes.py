"""GPU parity on seeded random shapes: batch size, group size, partition size, page size, cache
dtype and length mix drawn per case; adr_decode_step against the fp64 oracle's append and attention
(pools bit for bit, outputs within the floating-point gate), every kernel that serves the shape."""
import types

import numpy as np
import pytest
import torch

import oracle
import paper_2503_20552_amd as adr
import workloads as W
from gpu_util import compare, dev, say

pytestmark = pytest.mark.gpu

KERNELS = {"valu": adr.KERNEL_VALU, "mfma": adr.KERNEL_MFMA, "grid": adr.KERNEL_MFMA_GRID, "auto": adr.KERNEL_AUTO}


def draw_case(seed):
    rng = np.random.default_rng(9000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 8, 16]))
    B = int(rng.choice([1, 3, 17, 64, 200, 512]))
    page_size = int(rng.choice([16, 16, 32, 64]))
    part = int(rng.choice([0, 64, 128, 512]))
    fp8 = bool(rng.integers(0, 2))
    kind = int(rng.integers(0, 4))
    cap = max(8, 20000 // B)          # keeps a case's pool and the oracle's work small
    if kind == 0:
        lens = rng.integers(0, min(80, cap), size=B)
    elif kind == 1:
        lens = rng.integers(0, cap, size=B)
    elif kind == 2:
        lens = np.where(rng.random(B) < 0.1, rng.integers(cap, 4 * cap, size=B), rng.integers(0, 30, size=B))
    else:
        lens = np.full(B, int(rng.integers(1, cap)))
    lens = lens.astype(np.int32)
    if lens.max() == 0:
        lens[0] = 5
    return dict(Hkv=Hkv, G=G, B=B, page_size=page_size, part=part, fp8=fp8, lens=lens)


@pytest.mark.parametrize("seed", range(36))
def test_random_shape(seed):
    c = draw_case(seed)
    Hq, Hkv, d = c["G"] * c["Hkv"], c["Hkv"], 128
    lens_after = c["lens"]
    wl = W.Workload(96, "random", B=c["B"], Hq=Hq, Hkv=Hkv, d=d, lengths="given", page_size=c["page_size"])
    mb = W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=seed, lens_before=np.maximum(lens_after - 1, 0))
    positions = (lens_after - 1).astype(np.int32)
    part = c["part"]
    say("random shape %d: B=%d Hq=%d Hkv=%d page=%d part=%d fp8=%s tokens=%d" % (
        seed, c["B"], Hq, Hkv, c["page_size"], part, c["fp8"], int(lens_after.sum())))
    max_len = int(lens_after.max())
    if c["fp8"]:
        k0, ks0 = W.quantize_pool_fp8(dev(mb.k_cache), mb.used)
        v0, vs0 = W.quantize_pool_fp8(dev(mb.v_cache), mb.used)
        kh, vh, ksh, vsh = (W.bits(t).copy() for t in (k0, v0, ks0, vs0))
        oracle.kv_append(kh, vh, W.bits(mb.k_new), W.bits(mb.v_new), mb.block_table, positions, k_scale=ksh, v_scale=vsh)
        ref, ref_lse, _ = oracle.decode_attention(W.bits(mb.q), kh, vh, mb.block_table, lens_after, wl.scale,
                                                  k_scale=ksh, v_scale=vsh)
    else:
        k0, v0, ks0, vs0 = dev(mb.k_cache), dev(mb.v_cache), None, None
        kh, vh = W.bits(mb.k_cache).copy(), W.bits(mb.v_cache).copy()
        oracle.kv_append(kh, vh, W.bits(mb.k_new), W.bits(mb.v_new), mb.block_table, positions)
        ref, ref_lse, _ = oracle.decode_attention(W.bits(mb.q), kh, vh, mb.block_table, lens_after, wl.scale)
    ran = 0
    for name, flag in KERNELS.items():
        if name == "valu" and c["G"] > 8:
            continue
        if name == "grid" and c["fp8"]:
            continue
        kc, vc = k0.clone(), v0.clone()
        ks, vs = (ks0.clone(), vs0.clone()) if c["fp8"] else (None, None)
        out = torch.full((c["B"], Hq, d), float("nan"), dtype=torch.float32, device="cuda:0")
        lse = torch.full((c["B"], Hq), float("nan"), dtype=torch.float32, device="cuda:0")
        nbytes = adr.adr_decode_workspace_bytes(c["B"], Hq, d, max_len, part)
        ws = torch.full((max(nbytes, 4) // 4,), float("nan"), dtype=torch.float32, device="cuda:0") if nbytes else None
        adr.adr_decode_step(out, dev(mb.q), dev(mb.k_new), dev(mb.v_new), adr.KVCache(kc, vc, ks, vs),
                            dev(mb.block_table), dev(lens_after), wl.scale, max_len, part, ws, lse, flag)
        torch.cuda.synchronize()
        assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh), "pool after append, %s" % name
        if c["fp8"]:
            assert np.array_equal(W.bits(ks).view(np.uint32), ksh.view(np.uint32))
            assert np.array_equal(W.bits(vs).view(np.uint32), vsh.view(np.uint32))
        compare(out, lse, ref, ref_lse, what="random shape %d %s" % (seed, name))
        ran += 1
    assert ran >= 2
    assert adr.adr_stream_fault_count() == 0
