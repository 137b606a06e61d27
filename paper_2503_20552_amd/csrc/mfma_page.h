// Pieces shared by the two matrix-core decode kernels (d = 128, bf16 cache):
// per-page buffer descriptors, the K tile's LDS layout, and the per-page
// arithmetic S = K Q^T -> online softmax -> O += P V.  See decode_mfma.hip for
// the operand layouts.
#pragma once

#include "adr_device.h"

namespace adr {

constexpr int D = 128;

struct PageRegs {
    u32x4 v[4]; // natural rows, token 4j+u
};

constexpr int kTileBytes = kPageSize * D * 2; // one page of K for one kv-head
constexpr int kStages = 2;

// Cache policy of the K/V loads ("nt"): every byte is used once per pass, so it
// should not displace the block table, queries and partial results in the caches.
// Measured on MI355X: 6.9 TB/s instead of 6.1 TB/s for a bare ring of such loads.
constexpr int kStreamOnce = 2;

// Buffer descriptor of one cache page: base = the page, range = the page's
// bytes (reads past it return zero instead of touching memory), raw 32-bit
// addressing.  Built from wave-uniform values, so it lives in scalar registers
// and every load is "descriptor + 32-bit lane offset + scalar offset".
__device__ __forceinline__ __amdgpu_buffer_rsrc_t page_rsrc(const char *cache, int page,
                                                            uint32_t page_bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)(cache + (size_t)page * page_bytes), 0,
                                             (int)page_bytes, 0x00020000);
}

// The same with a range of its own: zero bytes make every lane's read out of range (zeros come
// back, and nothing is fetched).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t page_rsrc(const char *cache, int page,
                                                            uint32_t page_bytes, uint32_t range_bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)(cache + (size_t)page * page_bytes), 0,
                                             (int)range_bytes, 0x00020000);
}

// Issue the eight 16-byte loads of one page (this lane's share of K and V for
// one kv-head): four K loads that land in the LDS tile `ktile` (lane l of load
// i fills bytes [i*1024 + 16 l, +16) of the tile), four V loads into registers.
__device__ __forceinline__ void load_page(PageRegs &pr, char *ktile, __amdgpu_buffer_rsrc_t krsrc,
                                          __amdgpu_buffer_rsrc_t vrsrc, const uint32_t (&k_lane)[4],
                                          uint32_t v_lane, uint32_t tok_bytes)
{
    asm volatile("" ::: "memory"); // earlier reads of this tile stay ahead of the loads that refill it
#pragma unroll
    for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (__attribute__((address_space(3))) void *)(ktile + i * 1024),
                                                 16, k_lane[i], 0, 0, kStreamOnce);
#pragma unroll
    for (int u = 0; u < 4; ++u)
        pr.v[u] = __builtin_amdgcn_raw_buffer_load_b128(vrsrc, v_lane, u * tok_bytes, kStreamOnce);
    asm volatile("" ::: "memory");
}

// Wait until every vector-memory load except the newest group of eight has
// completed.  Loads return in order, so the page issued before that group is
// then whole: its K tile is in LDS (the compiler does not track loads that
// write LDS, hence the explicit wait) and its V rows are in registers.
__device__ __forceinline__ void wait_older_page()
{
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
}

// The running maximum of the online softmax only has to keep the weights in range, not to be
// the true maximum: it is moved up (and the accumulators rescaled, the expensive part of a
// step) only when a score exceeds it by more than this many powers of two, so weights reach
// 2^8 at most.  Numerator and denominator carry the same stale maximum, so the quotient and
// the log-sum-exp are unchanged.  With several heads per wave nearly every step of a short
// partition would otherwise rescale (the chance that one of four running maxima moves).
constexpr float kMaxSlack = 8.f;

struct WaveState {
    f32x4 o[8]; // O[head 4j+i][8r+e]
    float m;    // reference maximum of head r (same value in all four lane groups): >= true max - kMaxSlack
    float l;    // this lane's share of head r's denominator
};

// Eight OCP E4M3 bytes -> eight bf16 (exact: three mantissa bits fit in seven).  gfx950's
// v_cvt_scalef32_pk_bf16_fp8 turns two bytes into a bf16 pair in one instruction; the scale
// operand is 1, so nothing is rounded.
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ u32x4 fp8x8_to_bf16x8(u32x2 w)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    u32x4 r;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        r[2 * h] = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[h], 1.0f, false));
        r[2 * h + 1] = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[h], 1.0f, true));
    }
    return r;
}
#else // the host pass only parses device code
__device__ __forceinline__ u32x4 fp8x8_to_bf16x8(u32x2 w) { return u32x4{w[0], w[1], 0u, 0u}; }
#endif

// One page: S = K Q^T, online softmax, O += P V.
//   ka           A operand of QK^T (see decode_mfma.hip), one register group per step
//   score_scale  softmax scale * log2(e) (* the page's K scale for an fp8 cache)
//   p_scale      1, or the page's V scale for an fp8 cache: O += (P * p_scale) V
__device__ __forceinline__ void attend_page(WaveState &st, PageRegs &pg, const u32x4 (&ka)[4],
                                            const u32x4 (&qb)[4], float score_scale, float p_scale,
                                            int tok, int t1, int j)
{
    f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kk]),
                                                    __builtin_bit_cast(bf16x8, qb[kk]), s, 0, 0, 0);
    // tok = index of the first of this lane's four tokens (4j + i)
    const bool tail = tok - 4 * j + kPageSize > t1;
    float sc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sc[i] = s[i] * score_scale;
        if (tail && tok + i >= t1)
            sc[i] = -INFINITY;
    }
    if (tail) { // rows of tokens past the end may hold anything: keep them out of P*V
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (tok + u >= t1)
                pg.v[u] = u32x4{0u, 0u, 0u, 0u};
    }

    float bm = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
    bm = max_across_rows(bm);
    if (__any(bm > st.m + kMaxSlack)) {
        const float mn = fmaxf(st.m, bm);
        const float alpha = fast_exp2(st.m - mn);
        st.m = mn;
        st.l *= alpha;
        // O rows of this lane are heads 4j+i; their factors sit in lanes with r = 4j+i
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = __shfl(alpha, 4 * j + i);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                st.o[e][i] *= a;
        }
    }
    uint32_t ph[4], pl[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float pw = fast_exp2(sc[i] - st.m);
        st.l += pw;
        pw *= p_scale;
        ph[i] = __float_as_uint(pw) & 0xffff0000u;            // bf16 head (truncated)
        pl[i] = __float_as_uint(pw - __uint_as_float(ph[i])); // remainder, exact in fp32
    }
    u32x2 ah, al; // four bf16 each: element i <-> token 4j+i
    ah[0] = (ph[0] >> 16) | ph[1];
    ah[1] = (ph[2] >> 16) | ph[3];
    al[0] = (pl[0] >> 16) | (pl[1] & 0xffff0000u);
    al[1] = (pl[2] >> 16) | (pl[3] & 0xffff0000u);

#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        u32x2 vb;
        vb[0] = __builtin_amdgcn_perm(pg.v[1][e >> 1], pg.v[0][e >> 1], sel);
        vb[1] = __builtin_amdgcn_perm(pg.v[3][e >> 1], pg.v[2][e >> 1], sel);
        st.o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
            __builtin_bit_cast(s16x4, ah), __builtin_bit_cast(s16x4, vb), st.o[e], 0, 0, 0);
        st.o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
            __builtin_bit_cast(s16x4, al), __builtin_bit_cast(s16x4, vb), st.o[e], 0, 0, 0);
    }
}

} // namespace adr
