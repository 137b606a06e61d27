"""Pins for the fp64 oracle: every check here compares it with something that is
not its own formula -- closed forms, a dense numpy brute force, a library
attention routine, format tables, hand-indexed copies.  CPU only.

The paper (Sec. 2.1) prints no worked numerical example of attention, so there
are no printed values to pin against; these pins replace them.
"""
import math

import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st
from scipy.special import expit, logsumexp

import oracle
from oracle import dense_np
import workloads as W


def to_bits(x):
    """float array -> bf16 bit patterns (library cast, round-to-nearest-even)."""
    return W.bits(torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


def f64(bits):
    return dense_np.bf16_bits_to_f64(bits)


def tiny_problem(seed, B=3, Hq=8, Hkv=2, d=64, lens=(1, 17, 40), page_size=16, num_pages=40):
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens, dtype=np.int32)
    bt, num_pages, spare = W.deal_pages(lens, page_size, rng, fixed_pool_pages=num_pages)
    used = W.used_page_mask(bt, lens, page_size, num_pages)
    kc = W.bits(W.fill_pool_bf16(num_pages, page_size, Hkv, d, used, seed + 1))
    vc = W.bits(W.fill_pool_bf16(num_pages, page_size, Hkv, d, used, seed + 2))
    q = W.bits(W.randn_bf16((B, Hq, d), seed + 3))
    return q, kc, vc, bt, lens, 1.0 / math.sqrt(d)


# ---- (i) the five invariants ------------------------------------------------

def test_constant_v_returns_v():
    q, kc, vc, bt, lens, scale = tiny_problem(1)
    const = to_bits(np.float32(-1.375))
    vc[...] = const
    out, _, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    assert np.max(np.abs(out - (-1.375))) < 1e-15


def test_length_one_returns_its_v_and_score():
    q, kc, vc, bt, lens, scale = tiny_problem(2, lens=(1, 1, 1))
    out, lse, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    G = q.shape[1] // kc.shape[2]
    for b in range(3):
        page = bt[b, 0]
        for h in range(q.shape[1]):
            v0 = f64(vc[page, 0, h // G])
            k0 = f64(kc[page, 0, h // G])
            assert np.array_equal(out[b, h], v0)
            s0 = np.float64(np.float32(scale)) * np.dot(f64(q[b, h]), k0)
            assert abs(lse[b, h] - s0) < 1e-14 * max(1.0, abs(s0))


def test_weights_sum_to_one_and_are_a_distribution():
    q, kc, vc, bt, lens, scale = tiny_problem(3)
    for b in range(3):
        for h in (0, 5, 7):
            w = oracle.attention_weights(q, kc, vc, bt, lens, scale, b, h)
            assert w.shape == (lens[b],)
            assert np.all(w > 0) and abs(w.sum() - 1.0) < 1e-14


def test_physical_page_permutation_is_bit_invariant():
    q, kc, vc, bt, lens, scale = tiny_problem(4)
    out0, lse0, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    rng = np.random.default_rng(99)
    perm = rng.permutation(kc.shape[0])          # new id of old page p is perm[p]
    kc2 = np.empty_like(kc); vc2 = np.empty_like(vc)
    kc2[perm] = kc; vc2[perm] = vc
    bt2 = perm[bt].astype(np.int32)
    out1, lse1, _ = oracle.decode_attention(q, kc2, vc2, bt2, lens, scale)
    assert np.array_equal(out0, out1) and np.array_equal(lse0, lse1)


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 2), (8, 1)])
@pytest.mark.parametrize("d", [64, 128])
def test_dense_brute_force_agrees(Hq, Hkv, d):
    lens = (1, 15, 16, 17, 32, 33, 40)
    q, kc, vc, bt, lens, scale = tiny_problem(5 + Hkv + d, B=len(lens), Hq=Hq, Hkv=Hkv, d=d,
                                              lens=lens, num_pages=64)
    out, lse, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    kf = np.nan_to_num(f64(kc), nan=1e30)        # poison would blow up any stray read
    vf = np.nan_to_num(f64(vc), nan=1e30)
    out_d, lse_d = dense_np.decode_attention_dense(q, kf, vf, bt, lens, scale)
    assert np.max(np.abs(out - out_d)) < 1e-12
    assert np.max(np.abs(lse - lse_d)) < 1e-12


def test_library_attention_routine_agrees():
    """torch's scaled_dot_product_attention on CPU, float64, length-1 query."""
    q, kc, vc, bt, lens, scale = tiny_problem(11, B=2, Hq=8, Hkv=2, d=64, lens=(23, 37))
    out, _, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    G = 4
    for b in range(2):
        L = int(lens[b])
        Kd = dense_np.gather_dense(f64(kc), bt[b], L)      # [L,Hkv,d]
        Vd = dense_np.gather_dense(f64(vc), bt[b], L)
        Kt = torch.from_numpy(np.repeat(Kd, G, axis=1)).permute(1, 0, 2)   # [Hq,L,d]
        Vt = torch.from_numpy(np.repeat(Vd, G, axis=1)).permute(1, 0, 2)
        qt = torch.from_numpy(f64(q[b]))[:, None, :]                       # [Hq,1,d]
        ref = torch.nn.functional.scaled_dot_product_attention(
            qt, Kt, Vt, scale=float(np.float32(scale)))[:, 0, :].numpy()
        assert np.max(np.abs(out[b] - ref)) < 1e-12


# ---- (ii) closed forms -------------------------------------------------------

def test_zero_query_gives_mean_of_v_and_log_length():
    q, kc, vc, bt, lens, scale = tiny_problem(20)
    q[...] = 0
    out, lse, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    G = q.shape[1] // kc.shape[2]
    for b in range(3):
        L = int(lens[b])
        Vd = dense_np.gather_dense(f64(vc), bt[b], L)
        for h in range(q.shape[1]):
            assert np.max(np.abs(out[b, h] - Vd[:, h // G].mean(axis=0))) < 1e-14
            assert abs(lse[b, h] - math.log(L)) < 1e-14


def test_two_tokens_reduce_to_the_logistic_function():
    q, kc, vc, bt, lens, scale = tiny_problem(21, B=1, Hq=2, Hkv=2, d=64, lens=(2,))
    out, lse, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    page = bt[0, 0]
    for h in range(2):
        s = np.float64(np.float32(scale)) * (f64(kc[page, :2, h]) @ f64(q[0, h]))
        v0, v1 = f64(vc[page, 0, h]), f64(vc[page, 1, h])
        ref = v0 + expit(s[1] - s[0]) * (v1 - v0)
        assert np.max(np.abs(out[0, h] - ref)) < 1e-14
        assert abs(lse[0, h] - logsumexp(s)) < 1e-14


def test_dominant_key_selects_its_value():
    q, kc, vc, bt, lens, scale = tiny_problem(22, B=1, Hq=1, Hkv=1, d=64, lens=(30,))
    # integer-valued, exactly representable: q = e_0 * 8, k_t = 0 except token 7 has k[0] = 100
    q[...] = 0; kc[...] = 0
    q[0, 0, 0] = to_bits(np.float32(8.0))
    page, slot = bt[0, 0], 7
    kc[page, slot, 0, 0] = to_bits(np.float32(100.0))
    out, lse, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    # score gap = 800/8 = 100 -> the others weigh e^-100 each
    assert np.max(np.abs(out[0, 0] - f64(vc[page, slot, 0]))) < 1e-40 * 30 * 10 + 1e-16
    assert abs(lse[0, 0] - 100.0) < 1e-13


def test_shifting_all_keys_leaves_out_and_shifts_lse():
    rng = np.random.default_rng(23)
    q, kc, vc, bt, lens, scale = tiny_problem(23, B=1, Hq=4, Hkv=1, d=64, lens=(20,))
    # small integers are exact in bf16, and so are their sums below 256
    kc[...] = to_bits(rng.integers(-8, 9, size=kc.shape).astype(np.float32))
    q[...] = to_bits(rng.integers(-2, 3, size=q.shape).astype(np.float32))
    c = rng.integers(-4, 5, size=64).astype(np.float32)
    kc2 = to_bits((f64(kc) + c).astype(np.float32))
    assert np.array_equal(f64(kc2), f64(kc) + c)
    out0, lse0, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    out1, lse1, _ = oracle.decode_attention(q, kc2, vc, bt, lens, scale)
    assert np.max(np.abs(out0 - out1)) < 1e-13
    shift = np.float64(np.float32(scale)) * (f64(q[0]) @ c.astype(np.float64))
    assert np.max(np.abs((lse1 - lse0)[0] - shift)) < 1e-12


def test_gqa_equals_mha_with_replicated_kv_heads():
    q, kc, vc, bt, lens, scale = tiny_problem(24, Hq=8, Hkv=2)
    out_g, lse_g, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    kc_m = np.repeat(kc, 4, axis=2); vc_m = np.repeat(vc, 4, axis=2)
    out_m, lse_m, _ = oracle.decode_attention(q, kc_m, vc_m, bt, lens, scale)
    assert np.array_equal(out_g, out_m) and np.array_equal(lse_g, lse_m)


def test_padded_row_and_row_subset():
    q, kc, vc, bt, lens, scale = tiny_problem(25)
    lens0 = lens.copy(); lens0[1] = 0
    out, lse, _ = oracle.decode_attention(q, kc, vc, bt, lens0, scale)
    assert np.all(out[1] == 0) and np.all(np.isneginf(lse[1]))
    full, _, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    part, _, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale, rows=[2])
    assert np.array_equal(part[2], full[2]) and np.all(np.isnan(part[0]))


def test_strided_q_view_equals_contiguous():
    q, kc, vc, bt, lens, scale = tiny_problem(26)
    B, Hq, d = q.shape
    packed = np.zeros((B, (Hq + 4) * d), dtype=np.uint16)      # q followed by k,v as in a grouped buffer
    packed[:, :Hq * d] = q.reshape(B, -1)
    qv = packed[:, :Hq * d].reshape(B, Hq, d)
    assert not qv.flags["C_CONTIGUOUS"]
    a, la, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    b_, lb, _ = oracle.decode_attention(qv, kc, vc, bt, lens, scale)
    assert np.array_equal(a, b_) and np.array_equal(la, lb)


# ---- (iii) merge identity ----------------------------------------------------

def _split_and_merge(q, kc, vc, bt, lens, scale, cuts_per_row):
    """Attend each page-aligned piece separately (as its own request over a
    sliced block table), then merge with oracle.lse_merge."""
    B, Hq, d = q.shape
    ps = kc.shape[1]
    q_rows, bt_rows, len_rows, offsets = [], [], [], [0]
    for b in range(B):
        cuts = [0] + sorted(cuts_per_row[b]) + [int(lens[b])]
        n = 0
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            if hi <= lo:
                continue
            assert lo % ps == 0
            row = np.full(bt.shape[1], bt[b, 0], dtype=np.int32)
            pages = bt[b, lo // ps: -(-hi // ps)]
            row[:len(pages)] = pages
            q_rows.append(q[b]); bt_rows.append(row); len_rows.append(hi - lo); n += 1
        offsets.append(offsets[-1] + n)
    po, pl, _ = oracle.decode_attention(np.stack(q_rows), kc, vc, np.stack(bt_rows),
                                        np.asarray(len_rows, dtype=np.int32), scale)
    return oracle.lse_merge(po, pl, np.asarray(offsets, dtype=np.int32))


@settings(max_examples=25, deadline=None)
@given(st.lists(st.integers(0, 7), max_size=5), st.lists(st.integers(0, 3), max_size=3))
def test_split_then_merge_reproduces_unsplit(c0, c1):
    lens = (100, 49)
    q, kc, vc, bt, lens, scale = tiny_problem(30, B=2, Hq=4, Hkv=2, d=64, lens=lens, num_pages=24)
    cuts = [sorted({16 * c for c in c0 if 0 < 16 * c < 100}),
            sorted({16 * c for c in c1 if 0 < 16 * c < 49})]
    out, lse, _ = oracle.decode_attention(q, kc, vc, bt, lens, scale)
    mo, ml = _split_and_merge(q, kc, vc, bt, lens, scale, cuts)
    assert np.max(np.abs(out - mo)) < 1e-13 and np.max(np.abs(lse - ml)) < 1e-13


def test_merge_against_scipy_logsumexp_and_weighted_mean():
    rng = np.random.default_rng(31)
    P, heads, d = 7, 3, 5
    po = rng.standard_normal((P, heads, d)); pl = rng.standard_normal((P, heads)) * 4
    pl[2, 1] = -np.inf                               # an empty partition
    po[2, 1] = np.nan                                # whose payload must be ignored
    off = np.array([0, 3, 3, 7], dtype=np.int32)     # request 1 owns nothing
    out, lse = oracle.lse_merge(po, pl, off)
    for b, (lo, hi) in enumerate(zip(off[:-1], off[1:])):
        for h in range(heads):
            if hi == lo:
                assert np.all(out[b, h] == 0) and np.isneginf(lse[b, h]); continue
            ref_lse = logsumexp(pl[lo:hi, h])
            wts = np.exp(pl[lo:hi, h] - ref_lse)
            ref = np.nansum(wts[:, None] * np.where(wts[:, None] > 0, po[lo:hi, h], 0.0), axis=0)
            assert abs(lse[b, h] - ref_lse) < 1e-13 and np.max(np.abs(out[b, h] - ref)) < 1e-13


# ---- (vi) append --------------------------------------------------------------

def test_append_bf16_is_a_bit_copy_into_the_right_slot_only():
    wl = W.WORKLOADS[1]
    batch = W.make_batch(wl)
    kc, vc = W.bits(batch.k_cache).copy(), W.bits(batch.v_cache).copy()
    k_new, v_new = W.bits(batch.k_new), W.bits(batch.v_new)
    pos = batch.positions.copy(); pos[2] = -1                 # one skipped row
    k0, v0 = kc.copy(), vc.copy()
    oracle.kv_append(kc, vc, k_new, v_new, batch.block_table, pos)
    touched = np.zeros(kc.shape[:2], dtype=bool)
    for b in range(wl.B):
        if pos[b] < 0:
            continue
        page, slot = batch.block_table[b, pos[b] // 16], pos[b] % 16
        assert np.array_equal(kc[page, slot], k_new[b]) and np.array_equal(vc[page, slot], v_new[b])
        touched[page, slot] = True
    assert touched.sum() == 3
    assert np.array_equal(kc[~touched], k0[~touched]) and np.array_equal(vc[~touched], v0[~touched])


def test_append_rejects_out_of_table_position():
    wl = W.WORKLOADS[1]
    batch = W.make_batch(wl)
    kc, vc = W.bits(batch.k_cache).copy(), W.bits(batch.v_cache).copy()
    pos = batch.positions.copy(); pos[0] = batch.block_table.shape[1] * 16
    with pytest.raises(ValueError):
        oracle.kv_append(kc, vc, W.bits(batch.k_new), W.bits(batch.v_new), batch.block_table, pos)


# ---- (vii) fp8 ------------------------------------------------------------------

def test_fp8_e4m3_table_matches_format_definition_and_library():
    t = oracle.fp8_e4m3_decode_table()
    assert t[0] == 0 and t[0x80] == 0 and math.copysign(1, t[0x80]) == -1
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isnan(t).sum() == 2
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0
    assert [t[i] for i in range(1, 8)] == [i * 2.0 ** -9 for i in range(1, 8)]      # subnormals
    assert t[0x08] == 2.0 ** -6 and t[0x38] == 1.0 and t[0x3C] == 1.5
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).double().numpy()
    assert np.array_equal(np.nan_to_num(t, nan=7e7), np.nan_to_num(lib, nan=7e7))


def test_fp8_encoder_rounds_to_nearest_even_and_saturates():
    t = oracle.fp8_e4m3_decode_table()
    finite = np.sort(t[np.isfinite(t) & (t >= 0)])
    mids = (finite[:-1] + finite[1:]) / 2                      # exact ties
    codes = oracle.fp8_e4m3_encode(mids)
    assert np.all(codes % 2 == 0)                              # ties -> even mantissa
    assert np.all(np.abs(t[codes] - mids) == (finite[1:] - finite[:-1]) / 2)
    assert oracle.fp8_e4m3_encode(np.array([1e9, -1e9, 448.0, 464.0, 500.0])).tolist() == \
        [0x7E, 0xFE, 0x7E, 0x7E, 0x7E]
    rng = np.random.default_rng(40)
    x = (rng.standard_normal(4000) * 100).astype(np.float32)
    x = np.clip(x, -448, 448)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = oracle.fp8_e4m3_encode(x.astype(np.float64))
    same_value = t[mine] == t[lib]                             # +0/-0 may differ in sign bit only
    assert np.all(same_value)
    assert np.all(oracle.fp8_e4m3_encode(t[np.isfinite(t)]) == np.arange(256)[np.isfinite(t)])


def test_fp8_cache_attention_equals_bf16_attention_on_dequantised_values():
    """Values that are exact in both formats: the fp8 path must equal the bf16 path."""
    rng = np.random.default_rng(41)
    q, kc, vc, bt, lens, scale = tiny_problem(41, B=2, Hq=4, Hkv=2, d=64, lens=(19, 33))
    t = oracle.fp8_e4m3_decode_table()
    ok = np.nonzero(np.isfinite(t) & (np.abs(t) <= 4) & (np.abs(t) >= 2.0 ** -6) | (t == 0))[0]
    kb = rng.choice(ok, size=kc.shape).astype(np.uint8)
    vb = rng.choice(ok, size=vc.shape).astype(np.uint8)
    ks = (2.0 ** rng.integers(-2, 3, size=(kc.shape[0], 2))).astype(np.float32)   # power-of-two scales
    vs = (2.0 ** rng.integers(-2, 3, size=(kc.shape[0], 2))).astype(np.float32)
    k_deq = t[kb] * ks[:, None, :, None]; v_deq = t[vb] * vs[:, None, :, None]
    kc16, vc16 = to_bits(k_deq), to_bits(v_deq)
    assert np.array_equal(f64(kc16), k_deq)                   # 4 significant bits: exact in bf16
    o8, l8, _ = oracle.decode_attention(q, kb, vb, bt, lens, scale, k_scale=ks, v_scale=vs)
    o16, l16, _ = oracle.decode_attention(q, kc16, vc16, bt, lens, scale)
    assert np.array_equal(o8, o16) and np.array_equal(l8, l16)


def test_fp8_append_sets_scale_on_slot_zero_and_quantises_with_it():
    rng = np.random.default_rng(42)
    P, ps, Hkv, d, B = 6, 16, 2, 64, 3
    kb = np.full((P, ps, Hkv, d), 0x7F, dtype=np.uint8); vb = kb.copy()
    ks = np.full((P, Hkv), np.nan, dtype=np.float32); vs = ks.copy()
    ks[1] = [0.03125, 0.0625]; vs[1] = [0.00390625, 0.5]
    bt = np.array([[0, 5], [1, 5], [2, 3]], dtype=np.int32)
    pos = np.array([0, 5, 16], dtype=np.int32)                 # slot 0 of page 0; slot 5 of page 1; slot 0 of page 3
    k_new = to_bits(rng.standard_normal((B, Hkv, d))); v_new = to_bits(rng.standard_normal((B, Hkv, d)) * 3)
    oracle.kv_append(kb, vb, k_new, v_new, bt, pos, k_scale=ks, v_scale=vs)
    t = oracle.fp8_e4m3_decode_table()
    for (b, page, slot, fresh) in [(0, 0, 0, True), (1, 1, 5, False), (2, 3, 0, True)]:
        for h in range(Hkv):
            x = f64(k_new[b, h])
            if fresh:
                assert ks[page, h] == np.float32(np.float32(np.abs(x).max()) * np.float32(2.0 / 448.0))
            deq = t[kb[page, slot, h]] * np.float64(ks[page, h])
            # half a step of the format at the stored magnitude (3 mantissa bits), or saturation
            y = np.abs(x) / np.float64(ks[page, h])
            step = np.where(y < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(y, 1e-30))) - 3))
            bound = np.where(y > 448, np.inf, 0.5 * step * 1.0001 + 1e-6 * y) * np.float64(ks[page, h])
            assert np.all(np.abs(deq - x) <= bound)
            if fresh:                                           # headroom 2x: max lands at 224
                assert np.max(np.abs(t[kb[page, slot, h]])) == 224.0
    # a token that does not open a page leaves the page's scales as they were ...
    assert ks[1].tolist() == [0.03125, 0.0625] and vs[1].tolist() == [0.00390625, 0.5]
    # ... and what does not fit under the stored scale saturates at the largest finite code
    xv = f64(v_new[1, 0])
    over = np.abs(xv) / 0.00390625 > 464.0
    assert over.any() and np.all(np.abs(t[vb[1, 5, 0]][over]) == 448.0)
    assert np.all(np.sign(t[vb[1, 5, 0]][over]) == np.sign(xv[over]))
    untouched = np.ones((P, ps), dtype=bool)
    untouched[0, 0] = untouched[1, 5] = untouched[3, 0] = False
    assert np.all(kb[untouched] == 0x7F) and np.all(vb[untouched] == 0x7F)
    assert np.isnan(ks[[2, 4, 5]]).all()
