"""ctypes binding of include/adr.h.  Argument marshalling only."""
from __future__ import annotations

import contextlib
import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libadr.so")
_DEBUG_LIB_PATH = os.path.join(_HERE, "libadr_debug.so")   # the same sources with -DADR_DEBUG_BOUNDS

ADR_BF16, ADR_FP8_E4M3, ADR_F32 = 0, 1, 2
KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA, KERNEL_MFMA_GRID = 0, 1, 2, 3
PARTIALS_ONLY = 16
SINGLE_PARTITION_ITEMS = 32
WORKSPACE_READY = 64
DEBUG_EXPIRE_WAITS = 128


def GRID_CUS(n: int) -> int:
    """Flag bits that size the resident kernel's grid for n compute units (ADR_GRID_CUS)."""
    if not 0 < n < 4096:
        raise ValueError("compute units out of range")
    return n << 16


EXPORTS = ("adr_kv_append", "adr_decode_workspace_bytes", "adr_decode_attention", "adr_decode_attention_static",
           "adr_decode_step",
           "adr_decode_merge", "adr_lse_merge", "adr_probe_stream_read", "adr_probe_copy",
           "adr_stream_create_cu_mask", "adr_stream_destroy", "adr_stream_fault_count",
           "adr_decode_read_status", "adr_decode_kernel_choice", "adr_kernel_name", "adr_debug_bounds_status",
           "adr_offload_bound_mem", "adr_offload_bound_comp", "adr_offload_bound", "adr_need_offload",
           "adr_graph_capacity", "adr_pack_qkv", "adr_scatter_rows",
           "adr_graph_table_create", "adr_graph_table_capacity", "adr_graph_table_launch", "adr_graph_table_destroy",
           "adr_status_string", "adr_version")


class AdrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, adr_status_string(status), status))


class _CRequest(ctypes.Structure):
    _fields_ = [("max_token", ctypes.c_int64), ("used_token", ctypes.c_int64)]


class _CCache(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
                ("num_pages", ctypes.c_int), ("page_size", ctypes.c_int),
                ("Hkv", ctypes.c_int), ("d", ctypes.c_int), ("dtype", ctypes.c_int)]


class _CStepBuffers(ctypes.Structure):
    _fields_ = [("out", ctypes.c_void_p), ("out_dtype", ctypes.c_int), ("lse", ctypes.c_void_p),
                ("q", ctypes.c_void_p), ("q_row_stride", ctypes.c_int64),
                ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p), ("new_row_stride", ctypes.c_int64),
                ("caches", ctypes.POINTER(_CCache)), ("n_layers", ctypes.c_int),
                ("block_table", ctypes.c_void_p), ("max_pages_per_req", ctypes.c_int),
                ("seq_lens", ctypes.c_void_p), ("Hq", ctypes.c_int), ("scale", ctypes.c_float),
                ("max_seq_len", ctypes.c_int), ("partition_tokens", ctypes.c_int),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t), ("flags", ctypes.c_uint)]


class _CBoundsRecord(ctypes.Structure):
    _fields_ = [("count", ctypes.c_uint32), ("kind", ctypes.c_int32), ("row", ctypes.c_int32),
                ("index", ctypes.c_int32), ("value", ctypes.c_int32)]


_lib = None
_release_lib = None
_debug_lib = None


def library_path() -> str:
    return _LIB_PATH


@contextlib.contextmanager
def debug_library():
    """Inside the block every function of this module calls the debug build (libadr_debug.so)."""
    global _lib, _debug_lib
    if _debug_lib is None:
        if not os.path.exists(_DEBUG_LIB_PATH):
            raise ImportError("%s is missing: build it with `python -m paper_2503_20552_amd.build --debug`"
                              % _DEBUG_LIB_PATH)
        _debug_lib = _declare(ctypes.CDLL(_DEBUG_LIB_PATH))
    load_library()
    _lib = _debug_lib
    try:
        yield _debug_lib
    finally:
        _lib = _release_lib


def load_library():
    """Load libadr.so; fails loudly when it has not been built."""
    global _lib, _release_lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python -m paper_2503_20552_amd.build` "
            "(there is no fallback path)" % _LIB_PATH)
    _lib = _release_lib = _declare(ctypes.CDLL(_LIB_PATH))
    return _lib


def _declare(lib):
    """Argument and result types of every entry point."""
    vp, i32, i64, f32, sz, u32 = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float,
                                  ctypes.c_size_t, ctypes.c_uint)
    lib.adr_kv_append.restype = i32
    lib.adr_kv_append.argtypes = [ctypes.POINTER(_CCache), vp, vp, i64, vp, i32, vp, i32, vp]
    lib.adr_decode_workspace_bytes.restype = sz
    lib.adr_decode_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.adr_decode_attention.restype = i32
    lib.adr_decode_attention.argtypes = [vp, i32, vp, vp, i64, ctypes.POINTER(_CCache), vp, i32,
                                         vp, i32, i32, f32, i32, i32, vp, sz, u32, vp]
    lib.adr_decode_attention_static.restype = i32
    lib.adr_decode_attention_static.argtypes = [vp, i32, vp, vp, i64, ctypes.POINTER(_CCache), vp, i32,
                                                vp, i32, i32, f32, i32, i32, u32, vp]
    lib.adr_decode_step.restype = i32
    lib.adr_decode_step.argtypes = [vp, i32, vp, vp, i64, vp, vp, i64, ctypes.POINTER(_CCache), vp, i32,
                                    vp, i32, i32, f32, i32, i32, vp, sz, u32, vp]
    lib.adr_decode_merge.restype = i32
    lib.adr_decode_merge.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]
    lib.adr_lse_merge.restype = i32
    lib.adr_lse_merge.argtypes = [vp, i32, vp, vp, vp, vp, i32, i32, i32, vp]
    lib.adr_probe_stream_read.restype = i32
    lib.adr_probe_stream_read.argtypes = [vp, sz, vp, vp]
    lib.adr_probe_copy.restype = i32
    lib.adr_probe_copy.argtypes = [vp, vp, sz, vp]
    lib.adr_stream_create_cu_mask.restype = i32
    lib.adr_stream_create_cu_mask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_uint32), i32]
    lib.adr_stream_destroy.restype = i32
    lib.adr_stream_destroy.argtypes = [vp]
    f64 = ctypes.c_double
    lib.adr_offload_bound_mem.restype = f64
    lib.adr_offload_bound_mem.argtypes = [ctypes.POINTER(f64), ctypes.POINTER(f64), i32, f64, f64]
    lib.adr_offload_bound_comp.restype = f64
    lib.adr_offload_bound_comp.argtypes = [f64, f64]
    lib.adr_offload_bound.restype = f64
    lib.adr_offload_bound.argtypes = [f64, f64]
    lib.adr_need_offload.restype = i32
    lib.adr_need_offload.argtypes = [ctypes.POINTER(_CRequest), ctypes.POINTER(_CRequest), i32,
                                     ctypes.POINTER(_CRequest), i32, f64]
    lib.adr_pack_qkv.restype = i32
    lib.adr_pack_qkv.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, vp]
    lib.adr_scatter_rows.restype = i32
    lib.adr_scatter_rows.argtypes = [vp, i64, i32, vp, i64, vp, i32, i32, vp]
    lib.adr_graph_capacity.restype = i32
    lib.adr_graph_capacity.argtypes = [i32, i32, i32]
    lib.adr_stream_fault_count.restype = i32
    lib.adr_stream_fault_count.argtypes = [ctypes.POINTER(ctypes.c_uint64)]
    lib.adr_status_string.restype = ctypes.c_char_p
    lib.adr_status_string.argtypes = [i32]
    lib.adr_version.restype = i32
    lib.adr_version.argtypes = []
    lib.adr_decode_read_status.restype = i32
    lib.adr_decode_read_status.argtypes = [vp, sz, i32, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_uint32)]
    lib.adr_decode_kernel_choice.restype = i32
    lib.adr_decode_kernel_choice.argtypes = [ctypes.POINTER(_CCache), i32, i32, i32, i32, u32]
    lib.adr_kernel_name.restype = ctypes.c_char_p
    lib.adr_kernel_name.argtypes = [i32]
    lib.adr_debug_bounds_status.restype = i32
    lib.adr_debug_bounds_status.argtypes = [ctypes.POINTER(_CBoundsRecord), i32]
    lib.adr_graph_table_create.restype = i32
    lib.adr_graph_table_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(_CStepBuffers), i32, i32, vp]
    lib.adr_graph_table_capacity.restype = i32
    lib.adr_graph_table_capacity.argtypes = [vp, i32]
    lib.adr_graph_table_launch.restype = i32
    lib.adr_graph_table_launch.argtypes = [vp, i32, vp]
    lib.adr_graph_table_destroy.restype = i32
    lib.adr_graph_table_destroy.argtypes = [vp]
    return lib


def adr_stream_create_cu_mask(cu_bits) -> int:
    """A stream whose kernels run only on the compute units i with cu_bits[i] true; returns the
    raw hipStream_t handle (wrap it with torch.cuda.ExternalStream to use it from torch)."""
    bits = [bool(x) for x in cu_bits]
    words = (ctypes.c_uint32 * ((len(bits) + 31) // 32))()
    for i, on in enumerate(bits):
        if on:
            words[i // 32] |= 1 << (i % 32)
    handle = ctypes.c_void_p()
    _check(load_library().adr_stream_create_cu_mask(ctypes.byref(handle), words, len(words)),
           "adr_stream_create_cu_mask")
    return int(handle.value)


def adr_stream_destroy(handle: int) -> None:
    _check(load_library().adr_stream_destroy(ctypes.c_void_p(handle)), "adr_stream_destroy")


def adr_pack_qkv(dst: torch.Tensor, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, stream=None) -> None:
    """dst [B, >= (Hq+2Hkv)*d] bf16 <- q | k | v (each [B, heads, d], row-strided views allowed)."""
    qp, qs = _rows_view(q, "q")
    kp, ks = _rows_view(k, "k")
    vp_, vs = _rows_view(v, "v")
    B, Hq, d = q.shape
    Hkv = k.shape[1]
    if dst.dtype != torch.bfloat16 or dst.dim() != 2 or dst.shape[0] != B or dst.stride(1) != 1:
        raise ValueError("dst must be bf16 [B, width] with contiguous rows")
    if k.shape != v.shape or k.shape[0] != B or k.shape[2] != d or dst.shape[1] < (Hq + 2 * Hkv) * d:
        raise ValueError("shape mismatch")
    _check(load_library().adr_pack_qkv(dst.data_ptr(), dst.stride(0), qp, qs, kp, ks, vp_, vs, B, Hq, Hkv, d,
                                       _stream_handle(stream)), "adr_pack_qkv")


def adr_scatter_rows(dst: torch.Tensor, src: torch.Tensor, row_index: torch.Tensor, stream=None) -> None:
    """dst[row_index[i]] = src[i] for 2-D bf16 tensors with contiguous rows of equal width."""
    for t in (dst, src):
        if t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
            raise ValueError("dst and src must be bf16 [rows, width] with contiguous rows")
    if dst.shape[1] != src.shape[1] or row_index.dtype != torch.int32 or row_index.numel() != src.shape[0]:
        raise ValueError("shape mismatch")
    _check(load_library().adr_scatter_rows(dst.data_ptr(), dst.stride(0), dst.shape[0], src.data_ptr(),
                                           src.stride(0), row_index.data_ptr(), src.shape[0], src.shape[1],
                                           _stream_handle(stream)), "adr_scatter_rows")


def _requests(pairs):
    arr = (_CRequest * max(len(pairs), 1))()
    for i, (mx, used) in enumerate(pairs):
        arr[i].max_token, arr[i].used_token = int(mx), int(used)
    return arr


def adr_offload_bound_mem(hbm_prefill, bw_prefill, hbm_decode: float, bw_decode: float) -> float:
    n = len(hbm_prefill)
    if len(bw_prefill) != n:
        raise ValueError("one capacity and one bandwidth per prefill instance")
    f64n = ctypes.c_double * max(n, 1)
    return float(load_library().adr_offload_bound_mem(f64n(*hbm_prefill), f64n(*bw_prefill), n,
                                                      hbm_decode, bw_decode))


def adr_offload_bound_comp(b_max: float, b_tpot: float) -> float:
    return float(load_library().adr_offload_bound_comp(b_max, b_tpot))


def adr_offload_bound(ob_mem: float, ob_comp: float) -> float:
    return float(load_library().adr_offload_bound(ob_mem, ob_comp))


def adr_need_offload(req, local, offloaded, bound: float) -> bool:
    """req and the members of local / offloaded are (max_token, used_token) pairs."""
    rc = load_library().adr_need_offload(_requests([req]), _requests(local), len(local),
                                         _requests(offloaded), len(offloaded), bound)
    if rc < 0:
        raise AdrError(-rc, "adr_need_offload")
    return bool(rc)


def adr_graph_capacity(n: int, interval: int, max_capacity: int) -> int:
    return int(load_library().adr_graph_capacity(n, interval, max_capacity))


def adr_stream_fault_count() -> int:
    """Expired waits inside the resident-workgroup kernel on the current device (0 when healthy)."""
    n = ctypes.c_uint64(0)
    _check(load_library().adr_stream_fault_count(ctypes.byref(n)), "adr_stream_fault_count")
    return int(n.value)


def adr_decode_read_status(workspace: torch.Tensor, B: int, Hq: int, d: int, max_seq_len: int,
                           partition_tokens: int) -> int:
    """Waits that expired in calls on this workspace since its control area was last cleared."""
    n = ctypes.c_uint32(0)
    _check(load_library().adr_decode_read_status(workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                 B, Hq, d, int(max_seq_len), int(partition_tokens), ctypes.byref(n)),
           "adr_decode_read_status")
    return int(n.value)


def adr_decode_kernel_choice(cache: "KVCache", B: int, Hq: int, max_seq_len: int, partition_tokens: int,
                             flags: int = KERNEL_AUTO) -> int:
    cs = cache.c_struct()
    rc = load_library().adr_decode_kernel_choice(ctypes.byref(cs), B, Hq, int(max_seq_len), int(partition_tokens),
                                                 int(flags))
    if rc < 0:
        raise AdrError(-rc, "adr_decode_kernel_choice")
    return int(rc)


def adr_kernel_name(kernel: int) -> str:
    return load_library().adr_kernel_name(int(kernel)).decode()


def adr_debug_bounds_status(reset: bool = False) -> dict:
    """The debug build's record of out-of-range table entries and positions (see debug_library)."""
    rec = _CBoundsRecord()
    _check(load_library().adr_debug_bounds_status(ctypes.byref(rec), int(bool(reset))), "adr_debug_bounds_status")
    return {"count": int(rec.count), "kind": int(rec.kind), "row": int(rec.row), "index": int(rec.index),
            "value": int(rec.value)}


def adr_status_string(status: int) -> str:
    return load_library().adr_status_string(int(status)).decode()


def adr_version() -> int:
    return int(load_library().adr_version())


@dataclass
class KVCache:
    """One layer's paged cache: k, v [num_pages, page_size, Hkv, d] (bf16, or uint8 fp8 bytes
    with fp32 k_scale/v_scale [num_pages, Hkv])."""
    k: torch.Tensor
    v: torch.Tensor
    k_scale: Optional[torch.Tensor] = None
    v_scale: Optional[torch.Tensor] = None

    def c_struct(self) -> _CCache:
        num_pages, page_size, Hkv, d = self.k.shape
        if self.k.dtype == torch.bfloat16:
            dtype = ADR_BF16
        elif self.k.dtype == torch.uint8:
            dtype = ADR_FP8_E4M3
        else:
            raise TypeError("cache dtype must be bfloat16 or uint8 (fp8 bytes)")
        if self.v.shape != self.k.shape or self.v.dtype != self.k.dtype:
            raise ValueError("K and V caches differ in shape or dtype")
        if not (self.k.is_contiguous() and self.v.is_contiguous()):
            raise ValueError("caches must be contiguous")
        for s in (self.k_scale, self.v_scale):
            if s is not None and (s.dtype != torch.float32 or not s.is_contiguous()
                                  or tuple(s.shape) != (num_pages, Hkv)):
                raise ValueError("scales must be contiguous float32 [num_pages, Hkv]")
        return _CCache(self.k.data_ptr(), self.v.data_ptr(),
                       self.k_scale.data_ptr() if self.k_scale is not None else None,
                       self.v_scale.data_ptr() if self.v_scale is not None else None,
                       num_pages, page_size, Hkv, d, dtype)


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _rows_view(t: torch.Tensor, name: str):
    """[B, H, d] bf16 with heads and d contiguous; returns (ptr, row stride in elements)."""
    if t.dtype != torch.bfloat16 or t.dim() != 3:
        raise TypeError("%s must be bfloat16 [B, heads, d]" % name)
    if t.stride(2) != 1 or t.stride(1) != t.shape[2]:
        raise ValueError("%s: heads and d must be contiguous (only the row stride is free)" % name)
    return t.data_ptr(), t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1] * t.shape[2])


def _i32(t: torch.Tensor, name: str):
    if t.dtype != torch.int32 or not t.is_contiguous():
        raise TypeError("%s must be contiguous int32" % name)
    return t.data_ptr()


def _check(status: int, where: str):
    if status != 0:
        raise AdrError(status, where)


def adr_kv_append(cache: KVCache, k_new: torch.Tensor, v_new: torch.Tensor,
                  block_table: torch.Tensor, positions: torch.Tensor, stream=None) -> None:
    lib = load_library()
    cs = cache.c_struct()
    kp, kstride = _rows_view(k_new, "k_new")
    vp, vstride = _rows_view(v_new, "v_new")
    if kstride != vstride:
        raise ValueError("k_new and v_new must share one row stride")
    B = k_new.shape[0]
    if block_table.dim() != 2 or block_table.shape[0] != B or positions.shape != (B,):
        raise ValueError("block_table [B,max_pages] / positions [B] mismatch")
    _check(lib.adr_kv_append(ctypes.byref(cs), kp, vp, kstride, _i32(block_table, "block_table"),
                             block_table.shape[1], _i32(positions, "positions"), B,
                             _stream_handle(stream)), "adr_kv_append")


def adr_decode_workspace_bytes(B: int, Hq: int, d: int, max_seq_len: int,
                               partition_tokens: int) -> int:
    return int(load_library().adr_decode_workspace_bytes(B, Hq, d, max_seq_len, partition_tokens))


def _attention_args(out, q, cache, block_table, seq_lens, workspace, lse):
    qp, qstride = _rows_view(q, "q")
    B, Hq, d = q.shape
    if out.dtype == torch.bfloat16:
        odt = ADR_BF16
    elif out.dtype == torch.float32:
        odt = ADR_F32
    else:
        raise TypeError("out must be bfloat16 or float32")
    if tuple(out.shape) != (B, Hq, d) or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, Hq, d]")
    if lse is not None and (lse.dtype != torch.float32 or tuple(lse.shape) != (B, Hq)
                            or not lse.is_contiguous()):
        raise ValueError("lse must be contiguous float32 [B, Hq]")
    if block_table.dim() != 2 or block_table.shape[0] != B or seq_lens.shape != (B,):
        raise ValueError("block_table [B,max_pages] / seq_lens [B] mismatch")
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    return odt, (lse.data_ptr() if lse is not None else None), qp, qstride, B, Hq, ws_ptr, ws_bytes


def adr_decode_attention(out: torch.Tensor, q: torch.Tensor, cache: KVCache,
                         block_table: torch.Tensor, seq_lens: torch.Tensor, scale: float,
                         max_seq_len: int, partition_tokens: int = 0,
                         workspace: Optional[torch.Tensor] = None,
                         lse: Optional[torch.Tensor] = None, flags: int = KERNEL_AUTO,
                         stream=None) -> None:
    lib = load_library()
    cs = cache.c_struct()
    odt, lse_ptr, qp, qstride, B, Hq, ws_ptr, ws_bytes = _attention_args(out, q, cache, block_table, seq_lens,
                                                                         workspace, lse)
    _check(lib.adr_decode_attention(
        out.data_ptr(), odt, lse_ptr, qp, qstride,
        ctypes.byref(cs), _i32(block_table, "block_table"), block_table.shape[1],
        _i32(seq_lens, "seq_lens"), B, Hq, float(scale), int(max_seq_len), int(partition_tokens),
        ws_ptr, ws_bytes, int(flags), _stream_handle(stream)), "adr_decode_attention")


STATIC_SCRATCH_BYTES = 96 << 20


def adr_decode_attention_static(out: torch.Tensor, q: torch.Tensor, cache: KVCache,
                                block_table: torch.Tensor, seq_lens: torch.Tensor, scale: float,
                                max_seq_len: int, partition_tokens: int = 0,
                                lse: Optional[torch.Tensor] = None, flags: int = KERNEL_AUTO,
                                stream=None) -> None:
    """adr_decode_attention with the library's static device array as the workspace (no allocation)."""
    lib = load_library()
    cs = cache.c_struct()
    odt, lse_ptr, qp, qstride, B, Hq, _, _ = _attention_args(out, q, cache, block_table, seq_lens, None, lse)
    _check(lib.adr_decode_attention_static(
        out.data_ptr(), odt, lse_ptr, qp, qstride,
        ctypes.byref(cs), _i32(block_table, "block_table"), block_table.shape[1],
        _i32(seq_lens, "seq_lens"), B, Hq, float(scale), int(max_seq_len), int(partition_tokens),
        int(flags), _stream_handle(stream)), "adr_decode_attention_static")


def adr_decode_step(out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                    cache: KVCache, block_table: torch.Tensor, seq_lens: torch.Tensor, scale: float,
                    max_seq_len: int, partition_tokens: int = 0,
                    workspace: Optional[torch.Tensor] = None,
                    lse: Optional[torch.Tensor] = None, flags: int = KERNEL_AUTO,
                    stream=None) -> None:
    lib = load_library()
    cs = cache.c_struct()
    odt, lse_ptr, qp, qstride, B, Hq, ws_ptr, ws_bytes = _attention_args(out, q, cache, block_table, seq_lens,
                                                                         workspace, lse)
    kp, kstride = _rows_view(k_new, "k_new")
    vp, vstride = _rows_view(v_new, "v_new")
    if kstride != vstride:
        raise ValueError("k_new and v_new must share one row stride")
    if k_new.shape[0] != B or v_new.shape[0] != B:
        raise ValueError("k_new / v_new must have one row per request")
    _check(lib.adr_decode_step(
        out.data_ptr(), odt, lse_ptr, qp, qstride, kp, vp, kstride,
        ctypes.byref(cs), _i32(block_table, "block_table"), block_table.shape[1],
        _i32(seq_lens, "seq_lens"), B, Hq, float(scale), int(max_seq_len), int(partition_tokens),
        ws_ptr, ws_bytes, int(flags), _stream_handle(stream)), "adr_decode_step")


def adr_decode_merge(out: torch.Tensor, seq_lens: torch.Tensor, max_seq_len: int,
                     partition_tokens: int, workspace: Optional[torch.Tensor],
                     lse: Optional[torch.Tensor] = None, stream=None) -> None:
    lib = load_library()
    B, Hq, d = out.shape
    if out.dtype not in (torch.bfloat16, torch.float32) or not out.is_contiguous():
        raise TypeError("out must be contiguous bfloat16 or float32")
    odt = ADR_BF16 if out.dtype == torch.bfloat16 else ADR_F32
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(lib.adr_decode_merge(out.data_ptr(), odt, lse.data_ptr() if lse is not None else None,
                                _i32(seq_lens, "seq_lens"), B, Hq, d, int(max_seq_len),
                                int(partition_tokens), ws_ptr, ws_bytes, _stream_handle(stream)),
           "adr_decode_merge")


def adr_lse_merge(out: torch.Tensor, part_o: torch.Tensor, part_lse: torch.Tensor,
                  part_offsets: torch.Tensor, lse_out: Optional[torch.Tensor] = None,
                  stream=None) -> None:
    lib = load_library()
    B, heads, d = out.shape
    odt = ADR_BF16 if out.dtype == torch.bfloat16 else ADR_F32
    if out.dtype not in (torch.bfloat16, torch.float32) or not out.is_contiguous():
        raise TypeError("out must be contiguous bfloat16 or float32")
    if part_o.dtype != torch.float32 or part_lse.dtype != torch.float32:
        raise TypeError("partials must be float32")
    if not (part_o.is_contiguous() and part_lse.is_contiguous()):
        raise ValueError("partials must be contiguous")
    if part_o.dim() != 3 or tuple(part_o.shape[1:]) != (heads, d) \
            or tuple(part_lse.shape) != (part_o.shape[0], heads):
        raise ValueError("part_o [P,heads,d] / part_lse [P,heads] mismatch")
    if tuple(part_offsets.shape) != (B + 1,):
        raise ValueError("part_offsets must be int32 [B+1]")
    _check(lib.adr_lse_merge(out.data_ptr(), odt,
                             lse_out.data_ptr() if lse_out is not None else None,
                             part_o.data_ptr(), part_lse.data_ptr(),
                             _i32(part_offsets, "part_offsets"), B, heads, d,
                             _stream_handle(stream)), "adr_lse_merge")


def adr_probe_stream_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    n = src.numel() * src.element_size()
    if sink.numel() * sink.element_size() < 65536:
        raise ValueError("sink must hold at least 64 KiB")
    _check(load_library().adr_probe_stream_read(src.data_ptr(), n - n % 16, sink.data_ptr(),
                                                _stream_handle(stream)), "adr_probe_stream_read")


def adr_probe_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < n:
        raise ValueError("dst smaller than src")
    _check(load_library().adr_probe_copy(dst.data_ptr(), src.data_ptr(), n - n % 16,
                                         _stream_handle(stream)), "adr_probe_copy")


class GraphTable:
    """Pre-recorded decode steps for batch capacities interval, 2*interval, ..., max_capacity
    (adr_graph_table_*).  The tensors are the step's fixed buffers, sized for max_capacity rows; the
    caller overwrites their contents before each launch and keeps rows >= n padded (seq_lens 0)."""

    def __init__(self, out, q, k_new, v_new, caches, block_table, seq_lens, scale, max_seq_len, partition_tokens,
                 workspace, interval, max_capacity, capture_stream, lse=None, flags=KERNEL_AUTO):
        lib = load_library()
        odt, lse_ptr, qp, qstride, B, Hq, ws_ptr, ws_bytes = _attention_args(out, q, caches[0], block_table, seq_lens,
                                                                             workspace, lse)
        if B != max_capacity:
            raise ValueError("the buffers must hold max_capacity rows")
        kp, kstride = _rows_view(k_new, "k_new")
        vp_, vstride = _rows_view(v_new, "v_new")
        if kstride != vstride:
            raise ValueError("k_new and v_new must share one row stride")
        layer_structs = (_CCache * len(caches))(*[c.c_struct() for c in caches])
        desc = _CStepBuffers(out.data_ptr(), odt, lse_ptr, qp, qstride, kp, vp_, kstride, layer_structs, len(caches),
                             _i32(block_table, "block_table"), block_table.shape[1], _i32(seq_lens, "seq_lens"), Hq,
                             float(scale), int(max_seq_len), int(partition_tokens), ws_ptr, ws_bytes, int(flags))
        self._keep = (out, q, k_new, v_new, caches, block_table, seq_lens, workspace, lse)   # the graphs point into these
        self._handle = ctypes.c_void_p()
        self._lib = lib
        _check(lib.adr_graph_table_create(ctypes.byref(self._handle), ctypes.byref(desc), int(interval),
                                          int(max_capacity), _stream_handle(capture_stream)), "adr_graph_table_create")

    def capacity(self, n_rows: int) -> int:
        return int(self._lib.adr_graph_table_capacity(self._handle, int(n_rows)))

    def launch(self, n_rows: int, stream=None) -> None:
        _check(self._lib.adr_graph_table_launch(self._handle, int(n_rows), _stream_handle(stream)),
               "adr_graph_table_launch")

    def destroy(self) -> None:
        if self._handle:
            _check(self._lib.adr_graph_table_destroy(self._handle), "adr_graph_table_destroy")
            self._handle = ctypes.c_void_p()
