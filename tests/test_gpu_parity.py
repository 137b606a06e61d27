"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle
on the same seeded bytes.  Integer work (append slots, page gather) bit-exact;
floating point within |gpu-ref| <= 2e-3 + 1e-2*|ref| (bf16 K/V, fp32
accumulation), and max-abs <= 2e-3 on the fp32-output runs."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2503_20552_amd as adr
import workloads as W
from gpu_util import ATOL, compare, dev, gpu_attention, oracle_attention, say

pytestmark = pytest.mark.gpu

KERNELS = {"valu": adr.KERNEL_VALU, "mfma": adr.KERNEL_MFMA, "grid": adr.KERNEL_MFMA_GRID,
           "auto": adr.KERNEL_AUTO}


def small_case(seed, Hq, Hkv, d, lens, pool_pages=0):
    wl = W.Workload(99, "case", B=len(lens), Hq=Hq, Hkv=Hkv, d=d, lengths="given",
                    fixed_pool_pages=pool_pages)
    return W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=seed,
                        lens_before=np.asarray(lens, dtype=np.int32))


# ---- workload 1: append, then attend -------------------------------------------

@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_tiny_workload_append_then_attend(out_dtype):
    wl = W.WORKLOADS[1]
    bt = W.make_batch(wl)
    say("workload 1 append+attend out=%s" % out_dtype)
    kc, vc = dev(bt.k_cache), dev(bt.v_cache)
    cache = adr.KVCache(kc, vc)
    table, pos = dev(bt.block_table), dev(bt.positions)
    adr.adr_kv_append(cache, dev(bt.k_new), dev(bt.v_new), table, pos)
    torch.cuda.synchronize()
    # the oracle's append on a host copy; the whole pool, poison included, must match bit for bit
    kh, vh = W.bits(bt.k_cache).copy(), W.bits(bt.v_cache).copy()
    oracle.kv_append(kh, vh, W.bits(bt.k_new), W.bits(bt.v_new), bt.block_table, bt.positions)
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)

    out, lse = gpu_attention(dev(bt.q), kc, vc, table, dev(bt.seq_lens), wl.scale, out_dtype=out_dtype)
    ref, ref_lse, _ = oracle.decode_attention(W.bits(bt.q), kh, vh, bt.block_table, bt.seq_lens, wl.scale)
    max_abs, _ = compare(out, lse, ref, ref_lse, what="workload 1")
    if out_dtype == torch.float32:
        assert max_abs <= ATOL


def test_append_skips_negative_and_out_of_table_positions():
    b = small_case(1, 8, 2, 128, [5, 16, 31, 40])
    kc, vc = dev(b.k_cache), dev(b.v_cache)
    pos = b.positions.copy()
    pos[1] = -1
    pos[3] = b.block_table.shape[1] * 16 + 3        # beyond the row's table: skipped, not a fault
    say("append with skipped rows")
    adr.adr_kv_append(adr.KVCache(kc, vc), dev(b.k_new), dev(b.v_new), dev(b.block_table), dev(pos))
    torch.cuda.synchronize()
    kh, vh = W.bits(b.k_cache).copy(), W.bits(b.v_cache).copy()
    pos_ok = pos.copy(); pos_ok[3] = -1
    oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, pos_ok)
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)


def test_append_from_a_grouped_qkv_buffer():
    """q, k_new, v_new as views into one packed [B, (Hq+2Hkv)*d] buffer."""
    b = small_case(2, 8, 2, 128, [3, 47, 200])
    Hq, Hkv, d = 8, 2, 128
    packed = torch.cat([b.q.reshape(3, -1), b.k_new.reshape(3, -1), b.v_new.reshape(3, -1)], dim=1)
    packed = dev(packed)
    qv = packed[:, :Hq * d].view(3, Hq, d)
    kv = packed[:, Hq * d:(Hq + Hkv) * d].view(3, Hkv, d)
    vv = packed[:, (Hq + Hkv) * d:].view(3, Hkv, d)
    assert not qv.is_contiguous()
    kc, vc = dev(b.k_cache), dev(b.v_cache)
    say("grouped qkv views")
    adr.adr_kv_append(adr.KVCache(kc, vc), kv, vv, dev(b.block_table), dev(b.positions))
    out_v, lse_v = gpu_attention(qv, kc, vc, dev(b.block_table), dev(b.seq_lens), 0.09)
    out_c, lse_c = gpu_attention(dev(b.q), kc, vc, dev(b.block_table), dev(b.seq_lens), 0.09)
    assert torch.equal(out_v, out_c) and torch.equal(lse_v, lse_c)
    kh, vh = W.bits(b.k_cache).copy(), W.bits(b.v_cache).copy()
    oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, b.positions)
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)


# ---- shapes, tails, kernels, partitions ----------------------------------------------

LENS = [1, 2, 15, 16, 17, 31, 33, 63, 64, 65, 100, 257, 512, 513, 1000, 1499]


@pytest.mark.parametrize("kernel", ["valu", "mfma", "grid"])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 8, 128), (8, 2, 128), (8, 1, 128), (32, 8, 128),
                                      (4, 2, 128), (8, 8, 64), (8, 2, 64), (16, 2, 64)])
@pytest.mark.parametrize("partition_tokens", [0, 64, 512])
def test_attention_matches_oracle(kernel, Hq, Hkv, d, partition_tokens):
    if kernel in ("mfma", "grid") and d != 128:
        pytest.skip("the matrix-core kernel covers d = 128")
    b = small_case(10 + Hq + Hkv, Hq, Hkv, d, [L - 1 for L in LENS] + [0])
    seq = b.seq_lens.copy()
    seq[-1] = 0                                    # a padded row
    say("parity kernel=%s Hq=%d Hkv=%d d=%d part=%d" % (kernel, Hq, Hkv, d, partition_tokens))
    out, lse = gpu_attention(dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(b.block_table), dev(seq),
                             b.wl.scale, partition_tokens=partition_tokens, flags=KERNELS[kernel])
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, seq, b.wl.scale)
    max_abs, max_rel = compare(out, lse, ref, ref_lse, what="%s %d/%d/%d" % (kernel, Hq, Hkv, d))
    assert max_abs <= ATOL
    assert torch.all(out[-1] == 0) and torch.isneginf(lse[-1]).all()


@pytest.mark.parametrize("kernel", ["mfma", "grid"])
def test_groups_up_to_sixteen_on_the_matrix_cores(kernel):
    b = small_case(40, 32, 2, 128, [0, 16, 90, 700])
    say("G=16 mfma")
    out, lse = gpu_attention(dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(b.block_table),
                             dev(b.seq_lens), b.wl.scale, flags=KERNELS[kernel], partition_tokens=256)
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.wl.scale)
    assert compare(out, lse, ref, ref_lse, what="G=16")[0] <= ATOL


def test_bf16_output_is_the_rounded_fp32_output():
    b = small_case(41, 8, 2, 128, [99, 700, 15])
    args = (dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(b.block_table), dev(b.seq_lens), b.wl.scale)
    say("bf16 vs fp32 output")
    for part in (0, 128):
        o32, _ = gpu_attention(*args, partition_tokens=part)
        o16, _ = gpu_attention(*args, partition_tokens=part, out_dtype=torch.bfloat16)
        assert torch.equal(o32.to(torch.bfloat16), o16)


@pytest.mark.parametrize("kernel", ["valu", "mfma", "grid"])
def test_run_to_run_and_page_placement_invariance(kernel):
    b = small_case(42, 8, 2, 128, [700, 33, 1200, 5])
    table = dev(b.block_table); seq = dev(b.seq_lens); q = dev(b.q)
    say("determinism kernel=%s" % kernel)
    a1, l1 = gpu_attention(q, dev(b.k_cache), dev(b.v_cache), table, seq, b.wl.scale,
                           partition_tokens=256, flags=KERNELS[kernel])
    a2, l2 = gpu_attention(q, dev(b.k_cache), dev(b.v_cache), table, seq, b.wl.scale,
                           partition_tokens=256, flags=KERNELS[kernel])
    assert torch.equal(a1, a2) and torch.equal(l1, l2)
    rng = np.random.default_rng(7)
    perm = rng.permutation(b.num_pages)
    kc2 = torch.empty_like(b.k_cache); vc2 = torch.empty_like(b.v_cache)
    kc2[torch.from_numpy(perm)] = b.k_cache; vc2[torch.from_numpy(perm)] = b.v_cache
    a3, l3 = gpu_attention(q, dev(kc2), dev(vc2), dev(perm[b.block_table].astype(np.int32)), seq,
                           b.wl.scale, partition_tokens=256, flags=KERNELS[kernel])
    assert torch.equal(a1, a3) and torch.equal(l1, l3)


def test_max_seq_len_bound_truncates_rows():
    b = small_case(43, 8, 2, 128, [300, 40])
    say("max_seq_len truncation")
    out, lse = gpu_attention(dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(b.block_table),
                             dev(b.seq_lens), b.wl.scale, max_seq_len=128, partition_tokens=64)
    seq = np.minimum(b.seq_lens, 128).astype(np.int32)
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, seq, b.wl.scale)
    compare(out, lse, ref, ref_lse, what="truncated")


def test_out_of_range_page_ids_are_clamped_not_dereferenced():
    b = small_case(44, 8, 2, 128, [40, 40])
    table = b.block_table.copy()
    table[0, 1] = b.num_pages + 1000               # clamps to the last page
    table[1, 0] = -5                               # clamps to page 0
    say("clamped page ids")
    out, _ = gpu_attention(dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(table), dev(b.seq_lens), b.wl.scale)
    clamped = np.clip(table, 0, b.num_pages - 1).astype(np.int32)
    kc = torch.nan_to_num(b.k_cache.float(), nan=0.5).to(torch.bfloat16)
    vc = torch.nan_to_num(b.v_cache.float(), nan=0.5).to(torch.bfloat16)
    out2, _ = gpu_attention(dev(b.q), dev(kc), dev(vc), dev(clamped), dev(b.seq_lens), b.wl.scale)
    out3, _ = gpu_attention(dev(b.q), dev(kc), dev(vc), dev(table), dev(b.seq_lens), b.wl.scale)
    assert torch.equal(out2, out3)


# ---- the public merge ----------------------------------------------------------------

@pytest.mark.parametrize("d", [64, 128])
def test_lse_merge_matches_oracle(d):
    rng = np.random.default_rng(50 + d)
    counts = [0, 1, 2, 7, 33, 1, 0, 128]
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    P, heads = int(off[-1]), 5
    po = rng.standard_normal((P, heads, d)).astype(np.float32)
    pl = (rng.standard_normal((P, heads)) * 6).astype(np.float32)
    pl[3, 2] = -np.inf; po[3, 2] = np.nan                       # an empty partition with a poisoned payload
    pl[off[4]:off[5], 0] = -np.inf                              # a head with no mass at all
    say("lse_merge d=%d" % d)
    for dt in (torch.float32, torch.bfloat16):
        out = torch.full((len(counts), heads, d), float("nan"), dtype=dt, device="cuda:0")
        lse = torch.full((len(counts), heads), float("nan"), dtype=torch.float32, device="cuda:0")
        adr.adr_lse_merge(out, dev(po), dev(pl), dev(off), lse)
        torch.cuda.synchronize()
        ref, ref_lse = oracle.lse_merge(po.astype(np.float64), pl.astype(np.float64), off)
        o = out.float().cpu().numpy().astype(np.float64)
        tol = 1e-5 if dt == torch.float32 else 2.0 ** -8
        assert np.all(np.abs(o - ref) <= tol * (1 + np.abs(ref)))
        lg = lse.cpu().numpy().astype(np.float64)
        fin = np.isfinite(ref_lse)
        assert np.array_equal(np.isneginf(lg), ~fin)
        assert np.all(np.abs(lg[fin] - ref_lse[fin]) <= 1e-5 * (1 + np.abs(ref_lse[fin])))


def test_split_equals_unsplit_within_rounding():
    b = small_case(51, 32, 8, 128, [4000, 513, 77])
    args = (dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(b.block_table), dev(b.seq_lens), b.wl.scale)
    say("split vs unsplit")
    whole, lw = gpu_attention(*args)
    for part in (16, 512, 2048):
        split, ls = gpu_attention(*args, partition_tokens=part)
        assert (whole - split).abs().max().item() < 2e-5
        assert (lw - ls).abs().max().item() < 2e-5


@pytest.mark.parametrize("lo,hi,run", [(100, 165, 2), (225, 320, 4)])
@pytest.mark.parametrize("fp8", [False, True])
def test_many_items_are_handed_out_in_runs_of_partitions(lo, hi, run, fp8):
    """With tens of thousands of items the resident kernel takes runs of two or four partitions as one
    item and marks the other partitions of a run empty for the merge.  Lengths cross every boundary of
    partitions and runs; the merged result must be the oracle's, and the same as with the runs off."""
    rng = np.random.default_rng(77 + run)
    lens = rng.integers(lo, hi, size=512)
    lens[:12] = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 192, 0]
    items = int(np.sum(np.maximum(-(-(lens + 1) // 32), 1))) * 8
    assert items >= 8192 * run and (run == 4 or items < 8192 * 4), items   # the kernel's own thresholds
    b = small_case(61, 32, 8, 128, lens)
    say("runs of %d partitions, %d items, fp8=%s" % (run, items, fp8))
    if fp8:
        k8, ks = W.quantize_pool_fp8(b.k_cache, b.used)
        v8, vs = W.quantize_pool_fp8(b.v_cache, b.used)
        args = (dev(b.q), dev(k8), dev(v8), dev(b.block_table), dev(b.seq_lens), b.wl.scale)
        kw = dict(partition_tokens=32, k_scale=dev(ks), v_scale=dev(vs))
        ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), W.bits(k8), W.bits(v8), b.block_table, b.seq_lens,
                                                  b.wl.scale, k_scale=W.bits(ks), v_scale=W.bits(vs))
    else:
        args = (dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(b.block_table), dev(b.seq_lens), b.wl.scale)
        kw = dict(partition_tokens=32)
        ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.wl.scale)
    out, lse = gpu_attention(*args, flags=adr.KERNEL_MFMA, **kw)
    assert compare(out, lse, ref, ref_lse, what="runs of %d" % run)[0] <= ATOL
    single, lse1 = gpu_attention(*args, flags=adr.KERNEL_MFMA | adr.SINGLE_PARTITION_ITEMS, **kw)
    assert compare(single, lse1, ref, ref_lse, what="single-partition items")[0] <= ATOL
    assert not torch.equal(out, single)          # the two really took different routes
    assert (out - single).abs().max().item() < 2e-5


@pytest.mark.parametrize("fp8", [False, True])
def test_batches_of_more_than_512_rows_on_the_resident_kernel(fp8):
    """The resident kernel's length scan holds 512 rows; 1 100 rows go out as three launches."""
    rng = np.random.default_rng(91)
    lens = rng.integers(0, 90, size=1100)
    lens[[0, 511, 512, 1023, 1024, 1099]] = [200, 1, 130, 64, 0, 77]
    b = small_case(67, 8, 2, 128, lens)
    say("1100 rows on the resident kernel, fp8=%s" % fp8)
    if fp8:
        k8, ks = W.quantize_pool_fp8(b.k_cache, b.used)
        v8, vs = W.quantize_pool_fp8(b.v_cache, b.used)
        args = (dev(b.q), dev(k8), dev(v8), dev(b.block_table), dev(b.seq_lens), b.wl.scale)
        kw = dict(k_scale=dev(ks), v_scale=dev(vs))
        ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), W.bits(k8), W.bits(v8), b.block_table, b.seq_lens,
                                                  b.wl.scale, k_scale=W.bits(ks), v_scale=W.bits(vs))
    else:
        args = (dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(b.block_table), dev(b.seq_lens), b.wl.scale)
        kw = {}
        ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.wl.scale)
    for part in (0, 64):
        for out_dtype in (torch.float32, torch.bfloat16):
            out, lse = gpu_attention(*args, partition_tokens=part, flags=adr.KERNEL_MFMA, out_dtype=out_dtype, **kw)
            compare(out, lse, ref, ref_lse, what="1100 rows part=%d %s" % (part, out_dtype))


@pytest.mark.parametrize("kernel", ["valu", "mfma", "grid"])
def test_one_long_unsplit_row_among_short_ones(kernel):
    """A single pass over a 40 000-token row (2 500 pages through one item) next to tiny rows."""
    b = small_case(43, 8, 2, 128, [39999, 4, 299, 0])
    say("long unsplit row kernel=%s" % kernel)
    out, lse = gpu_attention(dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(b.block_table), dev(b.seq_lens),
                             b.wl.scale, flags=KERNELS[kernel])
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.wl.scale)
    assert compare(out, lse, ref, ref_lse, what="long row %s" % kernel)[0] <= ATOL


# ---- fp8-e4m3 cache -----------------------------------------------------------------

def fp8_case(seed, Hq, Hkv, d, lens):
    """A small case whose caches are quantised on the host (library casts only); the oracle
    reads the dequantised values, so only the attention arithmetic is under test."""
    b = small_case(seed, Hq, Hkv, d, lens)
    k8, ks = W.quantize_pool_fp8(b.k_cache, b.used)
    v8, vs = W.quantize_pool_fp8(b.v_cache, b.used)
    return b, k8, ks, v8, vs


@pytest.mark.parametrize("kernel", ["valu", "mfma", "auto"])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 8, 128), (8, 2, 128), (32, 8, 128), (16, 1, 128),
                                      (8, 8, 64), (8, 2, 64)])
@pytest.mark.parametrize("partition_tokens", [0, 64, 512])
def test_fp8_cache_attention_matches_oracle(kernel, Hq, Hkv, d, partition_tokens):
    if kernel == "mfma" and d != 128:
        pytest.skip("the matrix-core kernel covers d = 128")
    if kernel == "valu" and Hq // Hkv == 16:
        pytest.skip("the vector-ALU kernel covers groups of 1, 2, 4 and 8")
    b, k8, ks, v8, vs = fp8_case(60 + Hq + Hkv, Hq, Hkv, d, [L - 1 for L in LENS] + [0])
    seq = b.seq_lens.copy()
    seq[-1] = 0
    say("fp8 parity kernel=%s Hq=%d Hkv=%d d=%d part=%d" % (kernel, Hq, Hkv, d, partition_tokens))
    out, lse = gpu_attention(dev(b.q), dev(k8), dev(v8), dev(b.block_table), dev(seq), b.wl.scale,
                             partition_tokens=partition_tokens, flags=KERNELS[kernel],
                             k_scale=dev(ks), v_scale=dev(vs))
    ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), W.bits(k8), W.bits(v8), b.block_table, seq,
                                              b.wl.scale, k_scale=W.bits(ks), v_scale=W.bits(vs))
    max_abs, _ = compare(out, lse, ref, ref_lse, what="fp8 %s %d/%d/%d" % (kernel, Hq, Hkv, d))
    assert max_abs <= ATOL
    assert torch.all(out[-1] == 0) and torch.isneginf(lse[-1]).all()


def test_fp8_grid_kernel_is_reported_unsupported():
    b, k8, ks, v8, vs = fp8_case(61, 8, 2, 128, [40, 7])
    with pytest.raises(adr.AdrError):
        gpu_attention(dev(b.q), dev(k8), dev(v8), dev(b.block_table), dev(b.seq_lens), b.wl.scale,
                      flags=adr.KERNEL_MFMA_GRID, k_scale=dev(ks), v_scale=dev(vs))


@pytest.mark.parametrize("d", [64, 128])
def test_fp8_append_is_byte_exact_then_attend(d):
    """Append into an fp8 cache (slot 0 sets the page's scale, other slots reuse it and saturate),
    whole pool and both scale arrays byte for byte against the oracle's rule, then attend."""
    lens = [0, 1, 15, 16, 17, 32, 100, 255, 256]      # slot 0 (new page) and mid-page slots
    b, k8, ks, v8, vs = fp8_case(62 + d, 8, 2, d, lens)
    # a new token several times larger than the page's content: saturates where the scale is reused
    b.k_new[2] *= 6.0
    b.v_new[6] *= 6.0
    pos = b.positions.copy()
    pos[7] = -1                                        # a skipped row
    kd, vd, ksd, vsd = dev(k8), dev(v8), dev(ks), dev(vs)
    say("fp8 append d=%d" % d)
    adr.adr_kv_append(adr.KVCache(kd, vd, ksd, vsd), dev(b.k_new), dev(b.v_new), dev(b.block_table), dev(pos))
    torch.cuda.synchronize()
    kh, vh, ksh, vsh = (W.bits(t).copy() for t in (k8, v8, ks, vs))
    oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, pos, k_scale=ksh, v_scale=vsh)
    assert np.array_equal(W.bits(kd), kh) and np.array_equal(W.bits(vd), vh)
    assert np.array_equal(W.bits(ksd).view(np.uint32), ksh.view(np.uint32))
    assert np.array_equal(W.bits(vsd).view(np.uint32), vsh.view(np.uint32))

    seq = b.seq_lens.copy()
    seq[7] -= 1
    for kernel in ("valu", "mfma") if d == 128 else ("valu",):
        out, lse = gpu_attention(dev(b.q), kd, vd, dev(b.block_table), dev(seq), b.wl.scale,
                                 flags=KERNELS[kernel], k_scale=ksd, v_scale=vsd)
        ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), kh, vh, b.block_table, seq, b.wl.scale,
                                                  k_scale=ksh, v_scale=vsh)
        assert compare(out, lse, ref, ref_lse, what="fp8 append+attend %s" % kernel)[0] <= ATOL


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_fp8_every_finite_code_is_widened_exactly(kernel):
    """Rows of one token: out = the token's V (weight 1) and lse = its score, so each output
    element shows how one cache byte was decoded.  V carries all 254 finite codes, K of (row, head)
    carries one code in the dimension the one-hot query picks.  Neighbouring codes differ by 6 % or
    more; the bound is the 2^-15 the matrix-core kernel keeps of a weight (here the V scale)."""
    B, H, d = 32, 8, 128
    codes = np.arange(256, dtype=np.uint8)
    finite = ~np.isin(codes, [0x7F, 0xFF])
    num_pages = B
    k8 = np.zeros((num_pages, 16, H, d), dtype=np.uint8)
    v8 = np.zeros((num_pages, 16, H, d), dtype=np.uint8)
    pick = 5
    for row in range(B):
        for h in range(H):
            c = row * H + h
            k8[row, 0, h, pick] = c if finite[c] else 0x38           # 0x38 = 1.0
            vals = codes[(np.arange(d) + 128 * (h & 1)) % 256].copy()
            vals[~finite[vals]] = 0
            v8[row, 0, h, :] = vals
    rng = np.random.default_rng(3)
    ks = (0.5 + rng.random((num_pages, H))).astype(np.float32)
    vs = (0.5 + rng.random((num_pages, H))).astype(np.float32)
    q = torch.zeros((B, H, d), dtype=torch.bfloat16)
    q[:, :, pick] = 1.0
    table = np.arange(B, dtype=np.int32)[:, None]
    seq = np.ones(B, dtype=np.int32)
    say("fp8 code table kernel=%s" % kernel)
    out, lse = gpu_attention(dev(q), dev(k8), dev(v8), dev(table), dev(seq), 0.25, flags=KERNELS[kernel],
                             k_scale=dev(ks), v_scale=dev(vs))
    ref, ref_lse, _ = oracle.decode_attention(W.bits(q), k8, v8, table, seq, 0.25, k_scale=ks, v_scale=vs)
    g = out.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(g - ref) <= 4e-5 * np.abs(ref)), np.abs(g - ref).max()
    lg = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(lg - ref_lse) <= 4e-5 * np.abs(ref_lse) + 1e-30), np.abs(lg - ref_lse).max()


# ---- copies around the attention call -------------------------------------------------------------

def test_pack_qkv_then_views_feed_append_and_attention():
    """q, k, v grouped into one buffer by the library; the bytes equal the definition, and views of
    the packed buffer give the same append and attention as the separate tensors."""
    from oracle import glue_np
    b = small_case(80, 8, 2, 128, [3, 47, 200, 16])
    B, Hq, Hkv, d = 4, 8, 2, 128
    width = (Hq + 2 * Hkv) * d + 64                     # a padded row stride
    packed = torch.full((B, width), -1.0, dtype=torch.bfloat16, device="cuda:0")
    q_strided = dev(torch.cat([b.q.reshape(B, -1), torch.zeros(B, 8, dtype=torch.bfloat16)], 1))[:, :Hq * d].view(B, Hq, d)
    say("pack qkv")
    adr.adr_pack_qkv(packed, q_strided, dev(b.k_new), dev(b.v_new))
    torch.cuda.synchronize()
    want = glue_np.pack_qkv(W.bits(b.q), W.bits(b.k_new), W.bits(b.v_new), width=width,
                            fill=int(W.bits(torch.tensor([-1.0], dtype=torch.bfloat16))[0]))
    assert np.array_equal(W.bits(packed), want)
    qv = packed[:, :Hq * d].view(B, Hq, d)
    kv = packed[:, Hq * d:(Hq + Hkv) * d].view(B, Hkv, d)
    vv = packed[:, (Hq + Hkv) * d:(Hq + 2 * Hkv) * d].view(B, Hkv, d)
    kc1, vc1, kc2, vc2 = dev(b.k_cache), dev(b.v_cache), dev(b.k_cache), dev(b.v_cache)
    table, pos, seq = dev(b.block_table), dev(b.positions), dev(b.seq_lens)
    adr.adr_kv_append(adr.KVCache(kc1, vc1), kv, vv, table, pos)
    adr.adr_kv_append(adr.KVCache(kc2, vc2), dev(b.k_new), dev(b.v_new), table, pos)
    o1, l1 = gpu_attention(qv, kc1, vc1, table, seq, 0.09)
    o2, l2 = gpu_attention(dev(b.q), kc2, vc2, table, seq, 0.09)
    assert torch.equal(kc1.view(torch.int16), kc2.view(torch.int16)) and torch.equal(o1, o2) and torch.equal(l1, l2)


def test_scatter_rows_places_returned_rows_in_the_batch():
    from oracle import glue_np
    rng = np.random.default_rng(9)
    rows, n, width = 40, 17, 32 * 128
    dst = W.randn_bf16((rows, width), 5)
    src = W.randn_bf16((n, width), 6)
    index = rng.permutation(rows)[:n].astype(np.int32)
    index[3] = -1
    index[9] = rows + 5                                    # outside: skipped
    d_dst = dev(dst)
    say("scatter rows")
    adr.adr_scatter_rows(d_dst, dev(src), dev(index))
    torch.cuda.synchronize()
    assert np.array_equal(W.bits(d_dst), glue_np.scatter_rows(W.bits(dst), W.bits(src), index))


def test_graph_replay_matches_eager_on_every_replay():
    """Append + attention + merge of three layers recorded into one HIP graph; the per-step inputs
    live in fixed buffers.  Each replay is checked against the same step run eagerly, with eager
    work and synchronisation between the replays."""
    n_steps, n_layers, part = 4, 3, 512
    lens = np.asarray([700, 33, 1200, 5, 0, 511], dtype=np.int32)
    wl = W.Workload(99, "case", B=len(lens), Hq=8, Hkv=2, d=128, lengths="given")
    b = W.make_batch(wl, device="cpu", headroom_tokens=n_steps, seed_offset=70, lens_before=lens)
    table = dev(b.block_table)
    q = dev(b.q)
    k_new, v_new = dev(b.k_new), dev(b.v_new)
    lens0 = b.lens_before.copy()
    max_len = int(lens0.max()) + n_steps
    def fresh():
        return [adr.KVCache(dev(b.k_cache), dev(b.v_cache)) for _ in range(n_layers)]
    ws = torch.empty(max(adr.adr_decode_workspace_bytes(len(lens0), 8, 128, max_len, part), 256),
                     dtype=torch.uint8, device="cuda:0")
    out = torch.zeros((len(lens0), 8, 128), dtype=torch.float32, device="cuda:0")
    pos_buf = dev(lens0.astype(np.int32))
    seq_buf = dev((lens0 + 1).astype(np.int32))

    def step(caches):
        for c in caches:
            adr.adr_kv_append(c, k_new, v_new, table, pos_buf)
            adr.adr_decode_attention(out, q, c, table, seq_buf, b.wl.scale, max_len, part, ws, None,
                                     adr.KERNEL_MFMA)

    say("graph capture and replay")
    eager_caches, graph_caches = fresh(), fresh()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step(fresh())                        # warm the stream and the library before recording
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(graph_caches)
    for s in range(n_steps):
        pos_buf.copy_(dev((lens0 + s).astype(np.int32)))
        seq_buf.copy_(dev((lens0 + s + 1).astype(np.int32)))
        step(eager_caches)
        torch.cuda.synchronize()
        want = out.clone()
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), "replay %d differs from the eager step" % s
        for ce, cg in zip(eager_caches, graph_caches):
            assert torch.equal(ce.k.view(torch.int16), cg.k.view(torch.int16))
    assert adr.adr_stream_fault_count() == 0


def test_graph_recorded_at_a_capacity_serves_smaller_batches_with_padded_rows():
    """Sec. 3.2.2: graphs exist for batch capacities at an interval; a batch of n rows replays the
    smallest capacity that holds it, the surplus rows being padded (position < 0: no append;
    seq_len 0: zero output, no cache read).  One graph recorded at capacity 8 serves n = 8, 5, 1."""
    interval, cap_max, part = 4, 16, 256
    lens = np.asarray([700, 33, 1200, 5, 300, 511, 64, 17], dtype=np.int32)
    cap = adr.adr_graph_capacity(len(lens), interval, cap_max)
    assert cap == 8 and adr.adr_graph_capacity(5, interval, cap_max) == 8 and adr.adr_graph_capacity(1, interval, cap_max) == 4
    wl = W.Workload(99, "case", B=cap, Hq=8, Hkv=2, d=128, lengths="given")
    b = W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=71, lens_before=lens)
    table, q, k_new, v_new = dev(b.block_table), dev(b.q), dev(b.k_new), dev(b.v_new)
    max_len = int(lens.max()) + 1
    ws = torch.empty(max(adr.adr_decode_workspace_bytes(cap, 8, 128, max_len, part), 256), dtype=torch.uint8,
                     device="cuda:0")
    out = torch.zeros((cap, 8, 128), dtype=torch.float32, device="cuda:0")
    pos_buf, seq_buf = dev(lens.copy()), dev(lens + 1)
    kc, vc = dev(b.k_cache), dev(b.v_cache)
    cache = adr.KVCache(kc, vc)

    def step():
        adr.adr_kv_append(cache, k_new, v_new, table, pos_buf)
        adr.adr_decode_attention(out, q, cache, table, seq_buf, b.wl.scale, max_len, part, ws, None, adr.KERNEL_MFMA)

    say("graph at capacity 8, batches of 8, 5 and 1 rows")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    kh, vh = W.bits(b.k_cache).copy(), W.bits(b.v_cache).copy()
    oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, lens)
    for n in (8, 5, 1):
        pos = lens.copy(); seq = lens + 1
        pos[n:] = -1; seq[n:] = 0
        pos_buf.copy_(dev(pos)); seq_buf.copy_(dev(seq))
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        ref, _, _ = oracle.decode_attention(W.bits(b.q), kh, vh, b.block_table, seq.astype(np.int32), b.wl.scale)
        compare(out, None, ref, None, what="graph capacity 8, n=%d" % n)
        assert torch.all(out[n:] == 0)
    assert np.array_equal(W.bits(kc), kh) and np.array_equal(W.bits(vc), vh)   # padded rows appended nothing new


def test_resident_kernel_reports_no_expired_waits():
    """Runs after the cases above: none of the waves' bounded waits may have expired."""
    assert adr.adr_stream_fault_count() == 0


@pytest.mark.parametrize("bound", [None, 8192])
@pytest.mark.parametrize("kernel", ["grid", "valu", "mfma"])
def test_rows_of_many_partitions_and_a_loose_bound_on_the_lengths(kernel, bound):
    """The grids of the one-workgroup-per-item kernels are sized from the caller's bound on the lengths and
    give a row at most 33 workgroups per kv-head, which loop over the partitions of longer rows: rows of 1, 33,
    34, 67 and 70 partitions of 64 tokens, under the lengths' own maximum and under a bound twice as large
    (with the table padded to it)."""
    lens = [4479, 70, 2200, 1, 64 * 33, 64 * 33 + 1, 64 * 66 + 5, 0]
    b = small_case(123, 8, 2, 128, [max(L - 1, 0) for L in lens])
    seq = b.seq_lens.copy()
    seq[-1] = 0
    table = b.block_table
    if bound is not None:
        wide = np.zeros((table.shape[0], bound // 16), dtype=np.int32)
        wide[:, :table.shape[1]] = table
        table = wide
    say("many partitions, kernel=%s bound=%s" % (kernel, bound))
    out, lse = gpu_attention(dev(b.q), dev(b.k_cache), dev(b.v_cache), dev(table), dev(seq), b.wl.scale,
                             partition_tokens=64, flags=KERNELS[kernel], max_seq_len=bound)
    ref, ref_lse = oracle_attention(b.q, b.k_cache, b.v_cache, b.block_table, seq, b.wl.scale)
    max_abs, _ = compare(out, lse, ref, ref_lse, what="many partitions %s" % kernel)
    assert max_abs <= ATOL
