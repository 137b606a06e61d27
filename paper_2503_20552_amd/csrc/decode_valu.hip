// Decode attention with vector-ALU dot products (any supported shape, bf16 or
// fp8-e4m3 cache).
//
// One workgroup of 4 waves per (request, kv-head, partition).  Wave w streams
// pages w, w+4, ... of the partition.  A cache row (one token, one kv-head) is
// D bf16 = D/8 chunks of 16 bytes; lane l owns chunk l % (D/8) and token slot
// l / (D/8) of each 16-byte-per-lane load, so one load instruction fetches
// 64/(D/8) complete, contiguous rows.  All G q-heads of the group consume the
// same K/V registers.  Each (wave, token slot) keeps its own online-softmax
// state (running max, denominator, weighted V sum), merged once at the end:
// slots by wave shuffles, waves through LDS.
//
// An fp8 cache keeps the same lane <-> element mapping: a lane's eight elements
// are 8 bytes, widened by the hardware converter; the page's K scale multiplies
// the scores and its V scale the weights that enter the V sum.
#include "adr_device.h"

namespace adr {

// Eight cache elements of one lane as fp32.  Loaded with the non-temporal hint: each
// byte is used once per pass.
template <bool FP8> struct Row8;
template <> struct Row8<false> {
    u32x4 w;
    __device__ __forceinline__ void load(const void *cache, int64_t elem) { w = __builtin_nontemporal_load((const u32x4 *)((const uint16_t *)cache + elem)); }
    __device__ __forceinline__ void clear() { w = u32x4{0u, 0u, 0u, 0u}; }
    __device__ __forceinline__ void widen(float (&f)[8]) const
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = bf16_lo(w[e]);
            f[2 * e + 1] = bf16_hi(w[e]);
        }
    }
};
template <> struct Row8<true> {
    u32x2 w;
    __device__ __forceinline__ void load(const void *cache, int64_t elem) { w = __builtin_nontemporal_load((const u32x2 *)((const uint8_t *)cache + elem)); }
    __device__ __forceinline__ void clear() { w = u32x2{0u, 0u}; }
    __device__ __forceinline__ void widen(float (&f)[8]) const
    {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[h], false);
            const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[h], true);
            f[4 * h] = lo[0];
            f[4 * h + 1] = lo[1];
            f[4 * h + 2] = hi[0];
            f[4 * h + 3] = hi[1];
        }
    }
};

template <int D, int G, bool FP8>
__global__ __launch_bounds__(kThreads) void decode_valu_kernel(const DecodeParams p)
{
    constexpr int LPT = D / 8;          // lanes per token row
    constexpr int TPL = 64 / LPT;       // token rows per load instruction
    constexpr int U = kPageSize / TPL;  // load instructions per page

    const int Hkv = p.Hkv;
    // (an odd number of workgroups per row and kv-head: consecutive workgroups go to the compute
    // units in turn, and with an even number a row's few real ones fall on the same units row after row)
    const int stride = p.max_parts > 1 ? (p.max_parts | 1) : 1;
    const int kvh = blockIdx.x % Hkv;
    const int part = (blockIdx.x / Hkv) % stride;
    const int b = blockIdx.x / (Hkv * stride);

    const int L = min(p.seq_lens[b], p.max_seq_len);
    const int n_parts = parts_of(L, p.partition_tokens);
    if (part >= n_parts)
        return;
    const int t0 = p.partition_tokens > 0 ? part * p.partition_tokens : 0;
    const int t1 = p.partition_tokens > 0 ? min(L, t0 + p.partition_tokens) : L;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane % LPT;
    const int j = lane / LPT;

    // q for the G heads of this group, pre-multiplied by scale*log2(e)
    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const u32x4 w = *(const u32x4 *)(p.q + (int64_t)b * p.q_row_stride +
                                         (int64_t)(kvh * G + g) * D + c * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            qf[g][2 * e] = bf16_lo(w[e]) * p.scale_log2e;
            qf[g][2 * e + 1] = bf16_hi(w[e]) * p.scale_log2e;
        }
    }

    float m[G], l[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegBig;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            o[g][e] = 0.f;
    }

    const int64_t tok_stride = (int64_t)Hkv * D; // elements between tokens of a page
    const int32_t *bt = p.block_table + (int64_t)b * p.max_pages;
    const int pg_end = (t1 + kPageSize - 1) / kPageSize;

    for (int pg = t0 / kPageSize + wave; pg < pg_end; pg += kWaves) {
        const int page = pool_tile_checked(bt[pg >> p.page_shift], pg, p.num_pages, p.page_shift, p.bounds, b); // a 16-token tile
        const int64_t base = ((int64_t)page * kPageSize * Hkv + kvh) * D + c * 8;
        Row8<FP8> kr[U], vr[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            kr[u].load(p.k_cache, base + (u * TPL + j) * tok_stride);
#pragma unroll
        for (int u = 0; u < U; ++u)
            vr[u].load(p.v_cache, base + (u * TPL + j) * tok_stride);
        float k_scale = 1.f, v_scale = 1.f;
        if (FP8) {
            k_scale = p.k_scale[(int64_t)(page >> p.page_shift) * Hkv + kvh];
            v_scale = p.v_scale[(int64_t)(page >> p.page_shift) * Hkv + kvh];
        }

        float s[U][G];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[8];
            kr[u].widen(kf);
            const bool valid = pg * kPageSize + u * TPL + j < t1;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    dot = fmaf(qf[g][e], kf[e], dot);
                dot = group_sum<LPT>(dot);
                if (FP8)
                    dot *= k_scale;
                s[u][g] = valid ? dot : -INFINITY; // select, so garbage in unwritten slots never spreads
            }
            if (!valid)
                vr[u].clear();
        }
        float vf[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u)
            vr[u].widen(vf[u]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mn = m[g];
#pragma unroll
            for (int u = 0; u < U; ++u)
                mn = fmaxf(mn, s[u][g]);
            const float alpha = fast_exp2(m[g] - mn);
            m[g] = mn;
            float pw[U], ps = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                pw[u] = fast_exp2(s[u][g] - mn);
                ps += pw[u];
            }
            l[g] = l[g] * alpha + ps;
            if (FP8) {
#pragma unroll
                for (int u = 0; u < U; ++u)
                    pw[u] *= v_scale;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float acc = o[g][e] * alpha;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    acc = fmaf(pw[u], vf[u][e], acc);
                o[g][e] = acc;
            }
        }
    }

    // merge the TPL token slots of this wave (lanes j = 0..TPL-1 holding the same chunk c)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float M = m[g];
#pragma unroll
        for (int off = LPT; off < 64; off <<= 1)
            M = fmaxf(M, __shfl_xor(M, off));
        const float f = fast_exp2(m[g] - M);
        float ls = l[g] * f;
#pragma unroll
        for (int off = LPT; off < 64; off <<= 1)
            ls += __shfl_xor(ls, off);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = o[g][e] * f;
#pragma unroll
            for (int off = LPT; off < 64; off <<= 1)
                x += __shfl_xor(x, off);
            o[g][e] = x;
        }
        m[g] = M;
        l[g] = ls;
    }

    __shared__ float sm[kWaves * G], sl[kWaves * G], so[kWaves * G * D];
    if (j == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (c == 0) {
                sm[wave * G + g] = m[g];
                sl[wave * G + g] = l[g];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
                so[(wave * G + g) * D + c * 8 + e] = o[g][e];
        }
    }
    __syncthreads();
    combine_waves_and_store<D>(p, sm, sl, so, G, b, kvh, part, n_parts);
}

#define ADR_VALU_CASE(DD, GG)                                                                     \
    if (d == DD && G == GG) {                                                                     \
        if (fp8)                                                                                  \
            decode_valu_kernel<DD, GG, true><<<grid, kThreads, 0, stream>>>(p);                   \
        else                                                                                      \
            decode_valu_kernel<DD, GG, false><<<grid, kThreads, 0, stream>>>(p);                  \
        return hipGetLastError();                                                                 \
    }

hipError_t launch_decode_valu(const DecodeParams &p, int d, bool fp8, hipStream_t stream)
{
    const int G = p.G;
    const dim3 grid((unsigned)((int64_t)p.B * p.Hkv * (p.max_parts > 1 ? (p.max_parts | 1) : 1)));
    ADR_VALU_CASE(128, 1)
    ADR_VALU_CASE(128, 2)
    ADR_VALU_CASE(128, 4)
    ADR_VALU_CASE(128, 8)
    ADR_VALU_CASE(64, 1)
    ADR_VALU_CASE(64, 2)
    ADR_VALU_CASE(64, 4)
    ADR_VALU_CASE(64, 8)
    return hipErrorInvalidValue;
}

bool decode_valu_supports(int d, int G)
{
    return (d == 64 || d == 128) && (G == 1 || G == 2 || G == 4 || G == 8);
}

} // namespace adr
