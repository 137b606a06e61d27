"""Dense, unpaged numpy brute force for tiny inputs -- TEST INFRASTRUCTURE ONLY.

A second statement of the same definition as adr_oracle.c (Sec. 2.1 of the
paper: attention of the decode step's single query over the cached K and V),
written against materialised dense arrays with library calls, so that an
indexing or head-mapping slip in the C loops shows up as a disagreement.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits):
    """uint16 bf16 bit patterns -> float64 (exact)."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def gather_dense(cache_f64, block_table_row, L):
    """cache_f64 [pages,page_size,Hkv,d] -> the first L tokens [L,Hkv,d]."""
    page_size = cache_f64.shape[1]
    n_pages = -(-L // page_size)
    pages = np.asarray(block_table_row[:n_pages], dtype=np.int64)
    return cache_f64[pages].reshape(n_pages * page_size, *cache_f64.shape[2:])[:L]


def dense_attention(q_f64, K_f64, V_f64, scale):
    """q [Hq,d], K,V [L,Hkv,d] float64 -> (out [Hq,d], lse [Hq])."""
    Hq, d = q_f64.shape
    L, Hkv, _ = K_f64.shape
    G = Hq // Hkv
    K_rep = np.repeat(K_f64, G, axis=1)           # kv-head of q-head h is h // G
    V_rep = np.repeat(V_f64, G, axis=1)
    s = np.float64(np.float32(scale)) * np.einsum("hd,lhd->hl", q_f64, K_rep)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    Z = e.sum(axis=1, keepdims=True)
    out = np.einsum("hl,lhd->hd", e / Z, V_rep)
    return out, (m + np.log(Z))[:, 0]


def decode_attention_dense(q_bits, k_cache_f64, v_cache_f64, block_table, seq_lens, scale):
    """Whole batch through gather_dense + dense_attention."""
    B, Hq, d = q_bits.shape
    out = np.zeros((B, Hq, d))
    lse = np.full((B, Hq), -np.inf)
    qf = bf16_bits_to_f64(q_bits)
    for b in range(B):
        L = int(seq_lens[b])
        if L == 0:
            continue
        Kd = gather_dense(k_cache_f64, block_table[b], L)
        Vd = gather_dense(v_cache_f64, block_table[b], L)
        out[b], lse[b] = dense_attention(qf[b], Kd, Vd, scale)
    return out, lse
