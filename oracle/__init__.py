"""fp64 CPU oracle for paged decode attention -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares no code with the HIP library and never imports it.

`adr_oracle.c` holds the definition (two-pass softmax attention over gathered
pages, the append, the partition merge, the fp8 table); this module marshals
numpy arrays into it through ctypes.  `dense_np.py` is a second, unpaged numpy
brute force used on tiny inputs to pin the C code.

bf16 tensors are passed as numpy uint16 arrays holding the raw bits, fp8
tensors as uint8.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adr_oracle.c")
_LIB = os.path.join(_HERE, "libadr_oracle.so")

BF16 = 0
FP8_E4M3 = 1


PORTABLE_FLAGS = ["-O2"]
# The flags the CPU baseline is quoted with.  -ffp-contract=off keeps every product and sum
# rounded as written, so both builds give the same bits; the code is built on the machine
# that runs it, never shipped.
NATIVE_FLAGS = ["-O3", "-march=native", "-ffp-contract=off"]


def build(force: bool = False) -> str:
    """Compile adr_oracle.c with gcc (OpenMP) into libadr_oracle.so (portable code: the file may
    be built on one machine and loaded on another)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", *PORTABLE_FLAGS, "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def use_native_build(directory: str) -> str:
    """Build the same source for this machine's own CPU into `directory` and make this process
    use that build from now on (the benchmark's CPU-baseline leg calls it on the box it times)."""
    global _lib
    so = os.path.join(directory, "libadr_oracle_native.so")
    subprocess.check_call(["gcc", *NATIVE_FLAGS, "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall",
                           "-Wextra", "-o", so, _SRC, "-lm"])
    _lib = None
    _load(so)
    return " ".join(["gcc", *NATIVE_FLAGS, "-fopenmp"])


class _Cache(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
                ("num_pages", ctypes.c_int), ("page_size", ctypes.c_int),
                ("Hkv", ctypes.c_int), ("d", ctypes.c_int), ("dtype", ctypes.c_int)]


_lib = None


def _load(path=None):
    global _lib
    if _lib is None:
        # ADR_ORACLE_MUTANT names another build of the C file (a deliberately broken one, or one
        # with sanitizers); only the tests that check the pins against such builds set it.
        lib = ctypes.CDLL(path or os.environ.get("ADR_ORACLE_MUTANT") or build())
        lib.oracle_fp8_e4m3_decode.restype = ctypes.c_double
        lib.oracle_fp8_e4m3_decode.argtypes = [ctypes.c_uint8]
        lib.oracle_fp8_e4m3_encode.restype = ctypes.c_uint8
        lib.oracle_fp8_e4m3_encode.argtypes = [ctypes.c_double]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, a.dtype))
    return a


def _cache_struct(k_cache, v_cache, k_scale, v_scale):
    num_pages, page_size, Hkv, d = k_cache.shape
    if v_cache.shape != k_cache.shape:
        raise ValueError("K and V cache shapes differ")
    if k_cache.dtype == np.uint16:
        dtype = BF16
        keep = (_c(k_cache, np.uint16), _c(v_cache, np.uint16), None, None)
    elif k_cache.dtype == np.uint8:
        dtype = FP8_E4M3
        keep = (_c(k_cache, np.uint8), _c(v_cache, np.uint8),
                _c(k_scale, np.float32), _c(v_scale, np.float32))
        if keep[2].shape != (num_pages, Hkv) or keep[3].shape != (num_pages, Hkv):
            raise ValueError("scales must be [num_pages, Hkv]")
    else:
        raise TypeError("cache must be uint16 (bf16 bits) or uint8 (fp8 bytes)")
    s = _Cache(keep[0].ctypes.data, keep[1].ctypes.data,
               keep[2].ctypes.data if keep[2] is not None else None,
               keep[3].ctypes.data if keep[3] is not None else None,
               num_pages, page_size, Hkv, d, dtype)
    return s, keep


def _q_view(q):
    """q: uint16 [B, Hq, d]; the last two axes contiguous, any row stride."""
    if q.dtype != np.uint16 or q.ndim != 3:
        raise TypeError("q must be uint16 [B, Hq, d]")
    es = q.itemsize
    if q.strides[2] != es or q.strides[1] != q.shape[2] * es or q.strides[0] % es:
        q = np.ascontiguousarray(q)
    return q, q.strides[0] // es


def decode_attention(q, k_cache, v_cache, block_table, seq_lens, scale,
                     k_scale=None, v_scale=None, rows=None, num_threads=0):
    """softmax(scale * q K^T) V per (request, q-head), fp64.

    q [B,Hq,d] bf16 bits; caches [pages,page_size,Hkv,d] bf16 bits or fp8
    bytes (+ fp32 scales [pages,Hkv]); block_table int32 [B,max_pages];
    seq_lens int32 [B] (0 = padded row -> zeros, lse=-inf); `scale` is
    rounded to fp32 first, as the GPU receives it.  Returns
    (out [B,Hq,d] f64, lse [B,Hq] f64 natural log, threads_used).  With
    `rows`, only those requests are computed (others are left as NaN).
    """
    lib = _load()
    q, q_stride = _q_view(q)
    B, Hq, d = q.shape
    cs, keep = _cache_struct(k_cache, v_cache, k_scale, v_scale)
    if cs.d != d:
        raise ValueError("head dim mismatch")
    bt = _c(block_table, np.int32)
    sl = _c(seq_lens, np.int32)
    if bt.shape[0] != B or sl.shape != (B,):
        raise ValueError("block_table / seq_lens batch mismatch")
    out = np.full((B, Hq, d), np.nan, dtype=np.float64)
    lse = np.full((B, Hq), np.nan, dtype=np.float64)
    if rows is not None:
        rows = _c(np.asarray(rows, dtype=np.int32), np.int32)
    lib.oracle_decode_attention.restype = ctypes.c_int
    used = lib.oracle_decode_attention(
        _ptr(out), _ptr(lse), _ptr(q), ctypes.c_int64(q_stride), ctypes.byref(cs), _ptr(bt),
        ctypes.c_int(bt.shape[1]), _ptr(sl), ctypes.c_int(B), ctypes.c_int(Hq),
        ctypes.c_float(np.float32(scale)), _ptr(rows),
        ctypes.c_int(0 if rows is None else len(rows)), ctypes.c_int(num_threads))
    if used < 0:
        raise ValueError("oracle_decode_attention rejected its arguments (%d)" % used)
    del keep
    return out, lse, used


def attention_weights(q, k_cache, v_cache, block_table, seq_lens, scale, b, h,
                      k_scale=None, v_scale=None):
    """Normalised softmax weights of request b, q-head h: f64 [seq_lens[b]]."""
    lib = _load()
    q, q_stride = _q_view(q)
    B, Hq, d = q.shape
    cs, keep = _cache_struct(k_cache, v_cache, k_scale, v_scale)
    bt = _c(block_table, np.int32)
    sl = _c(seq_lens, np.int32)
    w = np.zeros(max(int(sl[b]), 1), dtype=np.float64)
    lib.oracle_attention_weights(
        _ptr(w), _ptr(q), ctypes.c_int64(q_stride), ctypes.byref(cs), _ptr(bt),
        ctypes.c_int(bt.shape[1]), _ptr(sl), ctypes.c_int(Hq),
        ctypes.c_float(np.float32(scale)), ctypes.c_int(b), ctypes.c_int(h))
    del keep
    return w[:int(sl[b])]


def _new_view(x):
    if x.dtype != np.uint16 or x.ndim != 3:
        raise TypeError("k_new/v_new must be uint16 [B, Hkv, d]")
    es = x.itemsize
    if x.strides[2] != es or x.strides[1] != x.shape[2] * es or x.strides[0] % es:
        x = np.ascontiguousarray(x)
    return x, x.strides[0] // es


def kv_append(k_cache, v_cache, k_new, v_new, block_table, positions,
              k_scale=None, v_scale=None):
    """Write each request's new K/V token into its page, IN PLACE.

    positions[b] is the token index written (the length before the append);
    negative skips the row.  bf16 caches: bit copy.  fp8 caches: quantised with
    the page's scale, which the token landing in slot 0 sets (see the C file).
    """
    lib = _load()
    num_pages, page_size, Hkv, d = k_cache.shape
    kn, ks = _new_view(k_new)
    vn, vs = _new_view(v_new)
    if ks != vs:
        vn = np.ascontiguousarray(vn)
        kn = np.ascontiguousarray(kn)
        ks = vs = Hkv * d
    bt = _c(block_table, np.int32)
    pos = _c(positions, np.int32)
    B = pos.shape[0]
    for a in (k_cache, v_cache):
        if not a.flags["C_CONTIGUOUS"] or not a.flags["WRITEABLE"]:
            raise ValueError("caches must be contiguous and writeable")
    if k_cache.dtype == np.uint16:
        rc = lib.oracle_kv_append_bf16(
            _ptr(k_cache), _ptr(v_cache), num_pages, page_size, Hkv, d, _ptr(kn), _ptr(vn),
            ctypes.c_int64(ks), _ptr(bt), ctypes.c_int(bt.shape[1]), _ptr(pos), ctypes.c_int(B))
    elif k_cache.dtype == np.uint8:
        for a in (k_scale, v_scale):
            if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"]:
                raise ValueError("scales must be contiguous float32")
        rc = lib.oracle_kv_append_fp8(
            _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), num_pages, page_size,
            Hkv, d, _ptr(kn), _ptr(vn), ctypes.c_int64(ks), _ptr(bt), ctypes.c_int(bt.shape[1]),
            _ptr(pos), ctypes.c_int(B))
    else:
        raise TypeError("cache dtype")
    if rc != 0:
        raise ValueError("oracle_kv_append: position or page out of range (%d)" % rc)


def lse_merge(part_o, part_lse, part_offsets):
    """Combine per-partition (normalised output, log-sum-exp) pairs, fp64.

    part_o [P,heads,d], part_lse [P,heads], part_offsets int32 [B+1] (CSR).
    Returns (out [B,heads,d], lse [B,heads]).
    """
    lib = _load()
    po = _c(np.asarray(part_o, dtype=np.float64), np.float64)
    pl = _c(np.asarray(part_lse, dtype=np.float64), np.float64)
    off = _c(np.asarray(part_offsets, dtype=np.int32), np.int32)
    B = off.shape[0] - 1
    _, heads, d = po.shape
    out = np.zeros((B, heads, d), dtype=np.float64)
    lse = np.zeros((B, heads), dtype=np.float64)
    lib.oracle_lse_merge(_ptr(out), _ptr(lse), _ptr(po), _ptr(pl), _ptr(off),
                         ctypes.c_int(B), ctypes.c_int(heads), ctypes.c_int(d))
    return out, lse


def fp8_e4m3_decode_table():
    """All 256 E4M3 codes decoded to fp64."""
    lib = _load()
    return np.array([lib.oracle_fp8_e4m3_decode(i) for i in range(256)], dtype=np.float64)


def fp8_e4m3_encode(x):
    """Round-to-nearest-even saturating encode of reals to E4M3 bytes."""
    lib = _load()
    flat = np.asarray(x, dtype=np.float64).ravel()
    return np.array([lib.oracle_fp8_e4m3_encode(float(v)) for v in flat],
                    dtype=np.uint8).reshape(np.shape(x))


def max_threads():
    return int(_load().oracle_max_threads())
