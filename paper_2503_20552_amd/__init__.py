"""MI355X-native paged decode attention: Python binding of the adr C ABI.

The binding only marshals arguments (torch tensors -> device pointers) into
libadr.so; every step of the path runs in the library's HIP kernels.  There is
no CPU fallback: if the library is missing, importing the binding's functions
raises.
"""
from .binding import (  # noqa: F401
    ADR_BF16, ADR_FP8_E4M3, ADR_F32, KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA, KERNEL_MFMA_GRID, PARTIALS_ONLY, SINGLE_PARTITION_ITEMS, WORKSPACE_READY, DEBUG_EXPIRE_WAITS, GRID_CUS,
    AdrError, KVCache, adr_kv_append, adr_decode_attention, adr_decode_attention_static, STATIC_SCRATCH_BYTES, adr_decode_step, adr_decode_workspace_bytes,
    adr_decode_merge, adr_lse_merge, adr_probe_stream_read, adr_probe_copy, adr_offload_bound_mem, adr_offload_bound_comp, adr_offload_bound, adr_need_offload,
    adr_graph_capacity, adr_pack_qkv, adr_scatter_rows, adr_stream_create_cu_mask, adr_stream_destroy, adr_stream_fault_count, adr_decode_read_status, adr_decode_kernel_choice, adr_kernel_name,
    adr_debug_bounds_status, debug_library, adr_status_string,
    adr_version,
    GraphTable, library_path, load_library,
)
