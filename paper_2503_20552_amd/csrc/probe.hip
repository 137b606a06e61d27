// Measurement aids: a streaming read and a plain copy, 16 bytes per lane.
#include "adr_device.h"

namespace adr {

__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *src, size_t n16, uint32_t *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i);
        const u32x4 b = __builtin_nontemporal_load(src + i + stride);
        const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride);
        const u32x4 d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n16; i += stride)
        acc ^= __builtin_nontemporal_load(src + i);
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    for (int off = 1; off < 64; off <<= 1)
        x ^= __shfl_xor(x, off);
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0)
        part[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0)
        sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

__global__ __launch_bounds__(256) void copy_kernel(u32x4 *dst, const u32x4 *src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

hipError_t launch_stream_read(const void *src, size_t bytes, void *sink, hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 256 * 16 - 1) / (256 * 16);
    if (blocks > 16384)
        blocks = 16384; // sink holds 4 bytes per block: 64 KiB
    if (blocks == 0)
        blocks = 1;
    stream_read_kernel<<<dim3((unsigned)blocks), 256, 0, stream>>>((const u32x4 *)src, n16,
                                                                  (uint32_t *)sink);
    return hipGetLastError();
}

hipError_t launch_copy(void *dst, const void *src, size_t bytes, hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 256 * 8 - 1) / (256 * 8);
    if (blocks > 65536)
        blocks = 65536;
    if (blocks == 0)
        blocks = 1;
    copy_kernel<<<dim3((unsigned)blocks), 256, 0, stream>>>((u32x4 *)dst, (const u32x4 *)src, n16);
    return hipGetLastError();
}

} // namespace adr
