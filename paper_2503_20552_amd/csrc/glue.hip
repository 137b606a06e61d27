// Copy kernels around the attention call (Sec. 3.2.1, 3.2.2): grouping q, k, v of a batch into one
// buffer that travels as one message, and placing rows of a result among the rows of a larger batch
// (how the decode side puts the remote attention outputs next to its local ones).  bf16 rows moved
// in 16-byte pieces, bit for bit.
#include "adr_device.h"

namespace adr {

struct PackParams {
    uint16_t *dst;
    const uint16_t *q, *k, *v;
    int64_t dst_stride, q_stride, k_stride, v_stride; // elements between request rows
    int q_elems, kv_elems;                            // Hq*d and Hkv*d
};

__global__ __launch_bounds__(256) void pack_qkv_kernel(const PackParams p)
{
    const int b = blockIdx.x;
    uint16_t *out = p.dst + (int64_t)b * p.dst_stride;
    const int total = p.q_elems + 2 * p.kv_elems;
    for (int i = threadIdx.x * 8; i < total; i += 256 * 8) {
        const uint16_t *src;
        if (i < p.q_elems)
            src = p.q + (int64_t)b * p.q_stride + i;
        else if (i < p.q_elems + p.kv_elems)
            src = p.k + (int64_t)b * p.k_stride + (i - p.q_elems);
        else
            src = p.v + (int64_t)b * p.v_stride + (i - p.q_elems - p.kv_elems);
        *(u32x4 *)(out + i) = *(const u32x4 *)src;
    }
}

struct ScatterParams {
    uint16_t *dst;
    const uint16_t *src;
    const int32_t *row_index;
    int64_t dst_stride, src_stride;
    int row_elems, dst_rows;
};

__global__ __launch_bounds__(256) void scatter_rows_kernel(const ScatterParams p)
{
    const int i = blockIdx.x;
    const int row = p.row_index[i];
    if (row < 0 || row >= p.dst_rows)
        return;
    const uint16_t *in = p.src + (int64_t)i * p.src_stride;
    uint16_t *out = p.dst + (int64_t)row * p.dst_stride;
    for (int e = threadIdx.x * 8; e < p.row_elems; e += 256 * 8)
        *(u32x4 *)(out + e) = *(const u32x4 *)(in + e);
}

hipError_t launch_pack_qkv(const PackParams &p, int B, hipStream_t stream)
{
    if (B == 0)
        return hipSuccess;
    pack_qkv_kernel<<<dim3(B), 256, 0, stream>>>(p);
    return hipGetLastError();
}

hipError_t launch_scatter_rows(const ScatterParams &p, int n, hipStream_t stream)
{
    if (n == 0)
        return hipSuccess;
    scatter_rows_kernel<<<dim3(n), 256, 0, stream>>>(p);
    return hipGetLastError();
}

} // namespace adr

#include "../../include/adr.h"

namespace {
bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
}

extern "C" {

int adr_pack_qkv(void *dst, int64_t dst_row_stride, const void *q, int64_t q_row_stride, const void *k,
                 int64_t k_row_stride, const void *v, int64_t v_row_stride, int B, int Hq, int Hkv, int d,
                 void *stream)
{
    if (!dst || !q || !k || !v)
        return ADR_ERR_NULL;
    if (B < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || (d % 8) != 0)
        return ADR_ERR_SHAPE;
    const int64_t qe = (int64_t)Hq * d, kve = (int64_t)Hkv * d;
    if (qe + 2 * kve > 0x7fffffffLL)
        return ADR_ERR_SHAPE;
    if (dst_row_stride < qe + 2 * kve || q_row_stride < qe || k_row_stride < kve || v_row_stride < kve)
        return ADR_ERR_SHAPE;
    if ((dst_row_stride | q_row_stride | k_row_stride | v_row_stride) % 8 != 0)
        return ADR_ERR_SHAPE;
    if (!aligned16(dst) || !aligned16(q) || !aligned16(k) || !aligned16(v))
        return ADR_ERR_SHAPE;
    adr::PackParams p;
    p.dst = (uint16_t *)dst;
    p.q = (const uint16_t *)q;
    p.k = (const uint16_t *)k;
    p.v = (const uint16_t *)v;
    p.dst_stride = dst_row_stride;
    p.q_stride = q_row_stride;
    p.k_stride = k_row_stride;
    p.v_stride = v_row_stride;
    p.q_elems = (int)qe;
    p.kv_elems = (int)kve;
    return adr::launch_pack_qkv(p, B, (hipStream_t)stream) == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
}

int adr_scatter_rows(void *dst, int64_t dst_row_stride, int dst_rows, const void *src, int64_t src_row_stride,
                     const int32_t *row_index, int n_rows, int row_elems, void *stream)
{
    if (!dst || !src || !row_index)
        return ADR_ERR_NULL;
    if (n_rows < 0 || dst_rows < 0 || row_elems <= 0 || (row_elems % 8) != 0)
        return ADR_ERR_SHAPE;
    if (dst_row_stride < row_elems || src_row_stride < row_elems || (dst_row_stride | src_row_stride) % 8 != 0)
        return ADR_ERR_SHAPE;
    if (!aligned16(dst) || !aligned16(src))
        return ADR_ERR_SHAPE;
    adr::ScatterParams p;
    p.dst = (uint16_t *)dst;
    p.src = (const uint16_t *)src;
    p.row_index = row_index;
    p.dst_stride = dst_row_stride;
    p.src_stride = src_row_stride;
    p.row_elems = row_elems;
    p.dst_rows = dst_rows;
    return adr::launch_scatter_rows(p, n_rows, (hipStream_t)stream) == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
}

} // extern "C"
