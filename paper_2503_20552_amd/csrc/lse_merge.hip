// Log-sum-exp merge of per-partition attention results.
//
// One group of d/4 threads per (request, head) row; each thread owns four
// consecutive output elements (16-byte loads of the fp32 partials).  One sweep
// over the row's partitions, sixteen at a time with all their loads issued before
// any is used, carrying a running maximum of the lse values (fixed order, so the
// result is the same from run to run).  When the attention pass left a non-zero
// expired-waits word in the call's status block, every row gets NaN instead.
#include "adr_device.h"

namespace adr {

template <int D>
__global__ __launch_bounds__(256) void lse_merge_kernel(const MergeParams p)
{
    constexpr int TPR = D / 4;        // threads per row
    constexpr int RPB = 256 / TPR;    // rows per block
    const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / TPR;
    const int col = (threadIdx.x % TPR) * 4;
    if (row >= (int64_t)p.B * p.heads)
        return;
    const int b = (int)(row / p.heads), h = (int)(row % p.heads);

    // The pass that wrote the partials reported a broken hand-shake between its waves: no row of
    // the call may pass as a result (rows with one partition included).
    if (p.status && p.status[kStatusExpiredWaits] != 0u) {
        const float nan = __builtin_nanf("");
        const int64_t off = row * D + col;
        if (p.out_f32) {
            *(f32x4 *)((float *)p.out + off) = f32x4{nan, nan, nan, nan};
        } else {
            *(u32x2 *)((uint16_t *)p.out + off) = u32x2{0x7fc07fc0u, 0x7fc07fc0u};
        }
        if (p.lse_out && col == 0)
            p.lse_out[row] = nan;
        return;
    }

    int first, count;
    if (p.part_offsets) {
        first = p.part_offsets[b];
        count = p.part_offsets[b + 1] - first;
    } else {
        const int L = max(min(p.seq_lens[b], p.max_seq_len), 0);
        count = parts_of(L, p.partition_tokens);
        first = b * p.max_parts;
        if (count <= 1)
            return; // the attention kernel already wrote this row's final result
    }

    constexpr int CH = 16;
    float top = -INFINITY, total = 0.f;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int i0 = 0; i0 < count; i0 += CH) {
        float ls[CH];
        f32x4 xs[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int64_t pr = (int64_t)(first + min(i0 + u, count - 1)) * p.heads + h;
            ls[u] = p.part_lse[pr];
            xs[u] = *(const f32x4 *)(p.part_o + pr * D + col);
        }
        float cm = -INFINITY;
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            if (i0 + u >= count)
                ls[u] = -INFINITY; // the clamped re-reads of the last partition carry no mass
            cm = fmaxf(cm, ls[u]);
        }
        const float nt = fmaxf(top, cm);
        if (nt > -INFINITY) {
            const float rs = fast_exp2((top - nt) * kLog2e); // 0 when nothing was seen before
            acc *= rs;
            total *= rs;
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const float w = fast_exp2((ls[u] - nt) * kLog2e);
                if (w > 0.f) { // an empty partition's payload is never used
                    acc += w * xs[u];
                    total += w;
                }
            }
            top = nt;
        }
    }
    const float inv = total > 0.f ? 1.f / total : 0.f;
    const int64_t off = row * D + col;
    if (p.out_f32) {
        *(f32x4 *)((float *)p.out + off) = acc * inv;
    } else {
        u32x2 w;
        w[0] = f32_to_bf16(acc[0] * inv) | (f32_to_bf16(acc[1] * inv) << 16);
        w[1] = f32_to_bf16(acc[2] * inv) | (f32_to_bf16(acc[3] * inv) << 16);
        *(u32x2 *)((uint16_t *)p.out + off) = w;
    }
    if (p.lse_out && col == 0)
        p.lse_out[row] = total > 0.f ? top + fast_log2(total) * kLn2 : -INFINITY;
}

hipError_t launch_lse_merge(const MergeParams &p, hipStream_t stream)
{
    const int64_t rows = (int64_t)p.B * p.heads;
    if (rows == 0)
        return hipSuccess;
    if (p.d == 128) {
        constexpr int RPB = 256 / 32;
        lse_merge_kernel<128><<<dim3((unsigned)((rows + RPB - 1) / RPB)), 256, 0, stream>>>(p);
    } else if (p.d == 64) {
        constexpr int RPB = 256 / 16;
        lse_merge_kernel<64><<<dim3((unsigned)((rows + RPB - 1) / RPB)), 256, 0, stream>>>(p);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace adr
