// Append of the decode step's new K/V token into its cache page.
#include "adr_device.h"

namespace adr {

// adr_decode_step: the append kernel runs right before the attention kernels of the same call,
// so its first workgroup also clears the call's control area for them.
__device__ __forceinline__ void clear_control(const AppendParams &p)
{
    if (p.clear_words && blockIdx.x == 0)
        for (int i = threadIdx.x; i < p.n_clear_words; i += blockDim.x)
            p.clear_words[i] = 0u;
}

// The page a row's token goes to, or -1 when the row is skipped (a padded row, a position past
// the row's table, a page id outside the pool; a debug build records the latter two, once per
// row: `report` is true in one thread of the row's workgroups).
__device__ __forceinline__ int append_page(const AppendParams &p, int b, int pos, bool report)
{
    if (pos < 0)
        return -1;
    if (pos / p.page_size >= p.max_pages) {
        if (report)
            record_out_of_bounds(p.bounds, 2, b, pos, p.max_pages * p.page_size);
        return -1;
    }
    const int page = p.block_table[(int64_t)b * p.max_pages + pos / p.page_size];
    if (page < 0 || page >= p.num_pages) {
        if (report)
            record_out_of_bounds(p.bounds, 3, b, pos / p.page_size, page);
        return -1;
    }
    return page;
}

// bf16 cache: one workgroup per request copies the Hkv*d bf16 of K and of V in
// 16-byte pieces.  The destination row of a token is contiguous.  The first pieces are
// read before the position and the page are looked up (they depend on neither), so the
// kernel is two memory round trips deep, not three.
__global__ __launch_bounds__(128) void kv_append_bf16_kernel(const AppendParams p)
{
    const int b = blockIdx.x;
    const int row = p.Hkv * p.d; // elements
    const int64_t src = (int64_t)b * p.new_row_stride;
    const int first = min((int)threadIdx.x * 8, row - 8);
    const u32x4 k0 = *(const u32x4 *)(p.k_new + src + first);
    const u32x4 v0 = *(const u32x4 *)(p.v_new + src + first);
    clear_control(p);
    const int pos = append_position(p, b);
    const int page = append_page(p, b, pos, threadIdx.x == 0);
    if (page < 0)
        return;
    const int64_t dst = ((int64_t)page * p.page_size + pos % p.page_size) * row;
    if ((int)threadIdx.x * 8 < row) {
        *(u32x4 *)((uint16_t *)p.k_cache + dst + first) = k0;
        *(u32x4 *)((uint16_t *)p.v_cache + dst + first) = v0;
    }
    for (int i = threadIdx.x * 8 + 128 * 8; i < row; i += 128 * 8) {
        *(u32x4 *)((uint16_t *)p.k_cache + dst + i) = *(const u32x4 *)(p.k_new + src + i);
        *(u32x4 *)((uint16_t *)p.v_cache + dst + i) = *(const u32x4 *)(p.v_new + src + i);
    }
}

// fp32 -> OCP E4M3 byte, round to nearest even, saturating at +-448, NaN -> 0x7F.
__device__ __forceinline__ uint32_t f32_to_e4m3(float x)
{
    const uint32_t u = __float_as_uint(x);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u)
        return 0x7Fu;
    const float ax = __uint_as_float(a);
    if (ax >= 464.0f) // halfway between 448 and the next (absent) step: everything above saturates
        return sign | 0x7Eu;
    uint32_t code;
    if (ax < 0.015625f) { // below 2^-6: subnormal codes, spacing 2^-9
        // adding 2^14 leaves ax/2^-9 rounded (to nearest even) in the low mantissa bits
        const float t = ax * 512.0f + 12582912.0f; // 1.5 * 2^23
        code = __float_as_uint(t) - 0x4B400000u;   // 0 .. 8 (8 = the smallest normal)
    } else {
        // keep 3 mantissa bits: round the fp32 mantissa at bit 20, nearest even
        const uint32_t rounded = a + 0x7FFFFu + ((a >> 20) & 1u);
        code = (rounded >> 20) - ((127u - 7u) << 3);
        if (code > 0x7Eu)
            code = 0x7Eu;
    }
    return sign | code;
}

// fp8 cache: one wave per (request, kv-head).  Lane i owns elements 2i, 2i+1
// (d = 128) or element i (d = 64).
template <int D>
__global__ __launch_bounds__(64) void kv_append_fp8_kernel(const AppendParams p)
{
    const int b = blockIdx.x / p.Hkv, h = blockIdx.x % p.Hkv;
    clear_control(p);
    const int pos = append_position(p, b);
    const int page = append_page(p, b, pos, threadIdx.x == 0 && h == 0);
    if (page < 0)
        return;
    const int slot = pos % p.page_size;
    constexpr int E = D / 64;
    const int lane = threadIdx.x;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const uint16_t *src = (which ? p.v_new : p.k_new) + (int64_t)b * p.new_row_stride + h * D;
        uint8_t *dst = (uint8_t *)(which ? p.v_cache : p.k_cache) +
                       (((int64_t)page * p.page_size + slot) * p.Hkv + h) * D;
        float *scales = which ? p.v_scale : p.k_scale;
        float x[E];
#pragma unroll
        for (int e = 0; e < E; ++e)
            x[e] = __uint_as_float((uint32_t)src[lane * E + e] << 16);
        float scale;
        if (slot == 0) {
            float amax = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e)
                amax = fmaxf(amax, fabsf(x[e]));
#pragma unroll
            for (int off = 1; off < 64; off <<= 1)
                amax = fmaxf(amax, __shfl_xor(amax, off));
            amax = fmaxf(amax, 9.5367431640625e-07f); // 2^-20
            scale = amax * (2.0f / 448.0f);
            if (lane == 0)
                scales[(int64_t)page * p.Hkv + h] = scale;
        } else {
            scale = scales[(int64_t)page * p.Hkv + h];
        }
        const float inv = 1.0f / scale;
        if (E == 2) {
            const uint32_t lo = f32_to_e4m3(x[0] * inv), hi = f32_to_e4m3(x[E - 1] * inv);
            *(uint16_t *)(dst + lane * 2) = (uint16_t)(lo | (hi << 8));
        } else {
            dst[lane] = (uint8_t)f32_to_e4m3(x[0] * inv);
        }
    }
}

hipError_t launch_kv_append(const AppendParams &p, bool fp8, hipStream_t stream)
{
    if (p.B == 0)
        return hipSuccess;
    if (!fp8)
        kv_append_bf16_kernel<<<dim3(p.B), 128, 0, stream>>>(p);
    else if (p.d == 128)
        kv_append_fp8_kernel<128><<<dim3(p.B * p.Hkv), 64, 0, stream>>>(p);
    else
        kv_append_fp8_kernel<64><<<dim3(p.B * p.Hkv), 64, 0, stream>>>(p);
    return hipGetLastError();
}

} // namespace adr
