// Decode attention with vector-ALU dot products (any supported shape).
//
// One workgroup of 4 waves per (request, kv-head, partition).  Wave w streams
// pages w, w+4, ... of the partition.  A cache row (one token, one kv-head) is
// D bf16 = D/8 chunks of 16 bytes; lane l owns chunk l % (D/8) and token slot
// l / (D/8) of each 16-byte-per-lane load, so one load instruction fetches
// 64/(D/8) complete, contiguous rows.  All G q-heads of the group consume the
// same K/V registers.  Each (wave, token slot) keeps its own online-softmax
// state (running max, denominator, weighted V sum), merged once at the end:
// slots by wave shuffles, waves through LDS.
#include "adr_device.h"

namespace adr {

template <int D, int G>
__global__ __launch_bounds__(kThreads) void decode_valu_kernel(const DecodeParams p)
{
    constexpr int LPT = D / 8;          // lanes per token row
    constexpr int TPL = 64 / LPT;       // token rows per load instruction
    constexpr int U = kPageSize / TPL;  // load instructions per page

    const int Hkv = p.Hkv;
    const int kvh = blockIdx.x % Hkv;
    const int part = (blockIdx.x / Hkv) % p.max_parts;
    const int b = blockIdx.x / (Hkv * p.max_parts);

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
    const uint16_t *kc = (const uint16_t *)p.k_cache;
    const uint16_t *vc = (const uint16_t *)p.v_cache;
    const int32_t *bt = p.block_table + (int64_t)b * p.max_pages;
    const int pg_end = (t1 + kPageSize - 1) / kPageSize;

    for (int pg = t0 / kPageSize + wave; pg < pg_end; pg += kWaves) {
        const int page = clamp_page(bt[pg], p.num_pages);
        const int64_t base = ((int64_t)page * kPageSize * Hkv + kvh) * D + c * 8;
        u32x4 kr[U], vr[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            kr[u] = *(const u32x4 *)(kc + base + (u * TPL + j) * tok_stride);
#pragma unroll
        for (int u = 0; u < U; ++u)
            vr[u] = *(const u32x4 *)(vc + base + (u * TPL + j) * tok_stride);

        float s[U][G];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                kf[2 * e] = bf16_lo(kr[u][e]);
                kf[2 * e + 1] = bf16_hi(kr[u][e]);
            }
            const bool valid = pg * kPageSize + u * TPL + j < t1;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    dot = fmaf(qf[g][e], kf[e], dot);
                dot = group_sum<LPT>(dot);
                s[u][g] = valid ? dot : -INFINITY; // select, so garbage in unwritten slots never spreads
            }
            if (!valid)
                vr[u] = u32x4{0u, 0u, 0u, 0u};
        }
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
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float acc = o[g][e] * alpha;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t w = vr[u][e >> 1];
                    acc = fmaf(pw[u], (e & 1) ? bf16_hi(w) : bf16_lo(w), acc);
                }
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
        decode_valu_kernel<DD, GG><<<grid, kThreads, 0, stream>>>(p);                             \
        return hipGetLastError();                                                                 \
    }

hipError_t launch_decode_valu(const DecodeParams &p, int d, hipStream_t stream)
{
    const int G = p.G;
    const dim3 grid((unsigned)((int64_t)p.B * p.Hkv * p.max_parts));
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
