"""The stored tiny case (tests/golden/tiny_case.json, written by tests/golden/make_tiny_case.py from
the oracle alone): the oracle must still give exactly these numbers, an unpaged numpy brute force
must agree with them, and the GPU path must match them within the path's tolerance."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import dense_np

HERE = os.path.dirname(os.path.abspath(__file__))


def load():
    c = json.load(open(os.path.join(HERE, "golden", "tiny_case.json")))
    u16 = lambda x: np.asarray(x, dtype=np.uint16)
    c["q"], c["k_new"], c["v_new"] = u16(c["q"]), u16(c["k_new"]), u16(c["v_new"])
    shape = (c["num_pages"], c["page_size"], c["Hkv"], c["d"])
    unhex = lambda h: np.asarray([int(h[i:i + 4], 16) for i in range(0, len(h), 4)], dtype=np.uint16).reshape(shape)
    c["k_cache_before"], c["v_cache_before"] = unhex(c["k_cache_before"]), unhex(c["v_cache_before"])
    c["block_table"] = np.asarray(c["block_table"], dtype=np.int32)
    c["positions"] = np.asarray(c["positions"], dtype=np.int32)
    c["seq_lens"] = np.asarray(c["seq_lens"], dtype=np.int32)
    c["out"] = np.asarray([[[float(x) for x in row] for row in req] for req in c["out"]])
    c["lse"] = np.asarray([[float(x) for x in row] for row in c["lse"]])
    return c


def test_oracle_reproduces_the_stored_case_exactly():
    c = load()
    k, v = c["k_cache_before"].copy(), c["v_cache_before"].copy()
    oracle.kv_append(k, v, c["k_new"], c["v_new"], c["block_table"], c["positions"])
    out, lse, _ = oracle.decode_attention(c["q"], k, v, c["block_table"], c["seq_lens"], c["scale"])
    assert np.array_equal(out, c["out"]) and np.array_equal(lse, c["lse"])


def test_stored_case_agrees_with_unpaged_brute_force():
    c = load()
    k, v = c["k_cache_before"].copy(), c["v_cache_before"].copy()
    oracle.kv_append(k, v, c["k_new"], c["v_new"], c["block_table"], c["positions"])
    out, lse = dense_np.decode_attention_dense(c["q"], dense_np.bf16_bits_to_f64(k), dense_np.bf16_bits_to_f64(v),
                                               c["block_table"], c["seq_lens"], c["scale"])
    assert np.allclose(out, c["out"], rtol=0, atol=1e-12)
    fin = np.isfinite(c["lse"])
    assert np.allclose(lse[fin], c["lse"][fin], rtol=0, atol=1e-12) and np.array_equal(np.isneginf(lse), ~fin)


@pytest.mark.gpu
def test_gpu_matches_the_stored_case():
    import paper_2503_20552_amd as adr
    from gpu_util import compare, gpu_attention
    c = load()
    bf = lambda a: torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).cuda()
    kc, vc = bf(c["k_cache_before"]), bf(c["v_cache_before"])
    table = torch.from_numpy(c["block_table"]).cuda()
    adr.adr_kv_append(adr.KVCache(kc, vc), bf(c["k_new"]), bf(c["v_new"]), table, torch.from_numpy(c["positions"]).cuda())
    out, lse = gpu_attention(bf(c["q"]), kc, vc, table, torch.from_numpy(c["seq_lens"]).cuda(), c["scale"])
    compare(out, lse, c["out"], c["lse"], what="stored tiny case")
