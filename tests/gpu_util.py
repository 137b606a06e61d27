"""Helpers shared by the GPU parity tests: run one decode step through the C
ABI on cuda:0 and through the fp64 oracle on the same bytes, and compare."""
from __future__ import annotations

import sys

import numpy as np
import torch

import oracle
import paper_2503_20552_amd as adr
import workloads as W

ATOL, RTOL = 2e-3, 1e-2   # bf16 K/V with fp32 accumulation: |gpu-ref| <= ATOL + RTOL*|ref|


def say(msg: str) -> None:
    """Name the case before each GPU step, flushed, so a dying box still tells which it was."""
    print("[gpu-case] " + msg, file=sys.stderr, flush=True)


def dev(x, dtype=None):
    t = torch.as_tensor(x)
    if dtype is not None:
        t = t.to(dtype)
    return t.to("cuda:0").contiguous()


def gpu_attention(q, k_cache, v_cache, block_table, seq_lens, scale, *, partition_tokens=0,
                  flags=adr.KERNEL_AUTO, out_dtype=torch.float32, max_seq_len=None,
                  k_scale=None, v_scale=None, want_lse=True):
    """All tensor arguments already on the device (block_table / seq_lens as int32)."""
    B, Hq, d = q.shape
    if max_seq_len is None:
        max_seq_len = int(seq_lens.max().item()) if B else 0
    out = torch.full((B, Hq, d), float("nan"), dtype=out_dtype, device=q.device)
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=q.device) if want_lse else None
    ws = None
    nbytes = adr.adr_decode_workspace_bytes(B, Hq, d, max_seq_len, partition_tokens)
    if nbytes:
        ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device=q.device)
    adr.adr_decode_attention(out, q, adr.KVCache(k_cache, v_cache, k_scale, v_scale), block_table,
                             seq_lens, scale, max_seq_len, partition_tokens, ws, lse, flags)
    torch.cuda.synchronize()
    return out, lse


def compare(out_gpu, lse_gpu, out_ref, lse_ref, rows=None, what=""):
    """Elementwise gate |gpu-ref| <= ATOL + RTOL*|ref|; returns (max_abs, max_rel)."""
    g = out_gpu.float().cpu().numpy().astype(np.float64)
    r = out_ref
    if rows is not None:
        g, r = g[rows], r[rows]
    assert np.isfinite(g).all(), what + ": non-finite values in the GPU output"
    err = np.abs(g - r)
    gate = ATOL + RTOL * np.abs(r)
    worst = np.unravel_index(np.argmax(err - gate), err.shape)
    assert (err <= gate).all(), "%s: |gpu-ref|=%.3e at %s (ref %.4f) exceeds %.3e" % (
        what, err[worst], worst, r[worst], gate[worst])
    big = np.abs(r) >= 1e-3
    max_rel = float((err[big] / np.abs(r[big])).max()) if big.any() else 0.0
    if lse_gpu is not None:
        lg = lse_gpu.cpu().numpy().astype(np.float64)
        lr = lse_ref
        if rows is not None:
            lg, lr = lg[rows], lr[rows]
        fin = np.isfinite(lr)
        assert np.array_equal(np.isneginf(lg), np.isneginf(lr)), what + ": lse -inf pattern"
        assert np.all(np.abs(lg[fin] - lr[fin]) <= ATOL + 1e-5 * np.abs(lr[fin])), \
            "%s: lse off by %.3e" % (what, np.abs(lg[fin] - lr[fin]).max())
    return float(err.max()), max_rel


def oracle_attention(q, k_cache, v_cache, block_table, seq_lens, scale, rows=None, **kw):
    out, lse, _ = oracle.decode_attention(W.bits(q), W.bits(k_cache), W.bits(v_cache),
                                          np.asarray(block_table, dtype=np.int32),
                                          np.asarray(seq_lens, dtype=np.int32), scale, rows=rows, **kw)
    return out, lse
