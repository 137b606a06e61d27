// Decode attention with the QK^T and PV contractions on the matrix cores
// (d = 128, bf16 cache, any group size G <= 16).
//
// One workgroup of 4 waves per (request, kv-head, partition); wave w streams
// pages w, w+4, ... .  A page holds exactly 16 tokens = one MFMA tile edge.
// Lane l is (r, j) = (l % 16, l / 16).
//
// QK^T  S[token][head] = K[16 x 128] * Q^T[128 x 16] as four
//       v_mfma_f32_16x16x32_bf16.  The A operand wants lane (r, j) to hold 16
//       bytes of token r -- sixteen different rows per quarter wave, a pattern
//       the vector memory path serves one lane at a time.  So the K tile takes
//       the coalesced route: four loads that each fetch four complete 256-byte
//       rows and deposit them directly in LDS (no VGPRs), and the operand is
//       then read from LDS.  Row t is stored with its sixteen 16-byte chunks
//       XOR-permuted by t (slot s holds chunk s ^ t), which makes the operand
//       reads -- sixteen rows, same chunk -- hit sixteen different bank groups.
//       Step kk, lane (r, j) contracts chunk kk*4 + j; Q^T (the B operand,
//       head r, loaded once) uses the same order.  Heads r >= G are zero
//       columns.  Each wave owns two such tiles (the page being consumed and
//       the page in flight).
//       Result layout: lane (r, j) holds S[token 4j+i][head r], i = 0..3.
// softmax  per lane over its 4 tokens, running max shared across the four
//       lane groups j by two wave shuffles; fp32 throughout, base 2.
// PV    O[head][dcol] += P[16 x 16 tokens] * V[16 tokens x 16 dcols], eight
//       v_mfma_f32_16x16x16_bf16 per page (one per e = 0..7, dcol = 8r + e).
//       The S layout above IS the A-operand layout (row = head r, k = token
//       4j+i), so P never moves between lanes.  P is split into a bf16 head
//       and a bf16 remainder (two MFMAs) so the weights keep ~16 significant
//       bits.  V is loaded in its natural layout -- lane (r, j), load u: the 16
//       bytes of token 4j+u at chunk r, i.e. four complete 256-byte rows per
//       instruction -- and the B operand (k = token 4j+u, n = r) for column
//       set e is assembled from those four registers with byte permutes.
//       Result layout: lane (r, j) holds O[head 4j+i][8r + e].
#include "mfma_page.h"

#include <algorithm>

namespace adr {

__device__ __forceinline__ void read_k_operand(u32x4 (&ka)[4], const char *ktile,
                                               const uint32_t (&k_read)[4])
{
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        ka[kk] = *(const u32x4 *)(ktile + k_read[kk]);
}

// Workgroups are numbered row by row: kv-head fastest (the heads of a page are read together),
// then the row's partitions, `stride` of them; a workgroup takes every stride-th partition of its
// row from its own on and leaves at once when the row has none for it.  The grid is sized from
// the caller's bound on the lengths, not from the lengths, so most workgroups may find nothing.
// Two things were measured on the 70B-shaped workload (1 712 items of 13 312 workgroups, 73 us):
// (1) the hardware hands consecutive workgroups to its compute units in turn, so when the number of
// workgroups per row divides the units evenly, a row's few real workgroups fall on the same units
// row after row: 123 us with 16 partitions per row in the grid, 152 us with 64.  The stride is
// therefore odd.  (2) Workgroups that find nothing still cost about a nanosecond each, and a loose
// bound makes tens of thousands of them: the stride stops at kGridStrideMax, and rows with more
// partitions (rare where this kernel is chosen) have their workgroups loop.
constexpr int kGridStrideMax = 33;
__host__ __device__ inline int grid_stride(int max_parts)
{
    const int n = max_parts < kGridStrideMax ? max_parts : kGridStrideMax;
    return n > 1 ? (n | 1) : n;
}

__global__ __launch_bounds__(kThreads) void decode_mfma_kernel(const DecodeParams p)
{
    const int Hkv = p.Hkv, G = p.G;
    const int stride = grid_stride(p.max_parts);
    const int kvh = blockIdx.x % Hkv;
    const int first_part = (blockIdx.x / Hkv) % stride;
    const int b = blockIdx.x / (Hkv * stride);

    const int L = max(min(p.seq_lens[b], p.max_seq_len), 0);
    const int n_parts = parts_of(L, p.partition_tokens);
    if (first_part >= n_parts)
        return;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15;
    const int j = lane >> 4;

    // B operand of QK^T: head r's query, chunk order matching the K loads
    u32x4 qb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        qb[kk] = u32x4{0u, 0u, 0u, 0u};
        if (r < G)
            qb[kk] = *(const u32x4 *)(p.q + (int64_t)b * p.q_row_stride +
                                      (int64_t)(kvh * G + r) * D + (kk * 4 + j) * 8);
    }

    // Byte offsets of this lane.
    //  K load i (to LDS): row t = 4i + j, slot r of that row, which holds chunk r ^ t.
    //  K operand read, step kk: row r, chunk kk*4 + j, which sits in slot (kk*4 + j) ^ r.
    //  V load u (to registers): row 4j + u, chunk r.
    const uint32_t tok_bytes = (uint32_t)Hkv * D * 2;
    uint32_t k_lane[4], k_read[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = 4 * i + j;
        k_lane[i] = (uint32_t)kvh * D * 2 + t * tok_bytes + ((r ^ t) * 16);
        k_read[i] = r * (D * 2) + (((i * 4 + j) ^ r) * 16);
    }
    const uint32_t v_lane = (uint32_t)kvh * D * 2 + 4 * j * tok_bytes + r * 16;
    const uint32_t page_bytes = kPageSize * tok_bytes;
    const char *kc = (const char *)p.k_cache;
    const char *vc = (const char *)p.v_cache;
    // The block table is read through the constant address space: its entries are
    // wave-uniform and never written while the kernel runs, so they arrive by
    // scalar loads and stay out of the vector-memory counter the waits rely on.
    typedef const __attribute__((address_space(4))) int32_t *table_ptr;
    table_ptr bt = (table_ptr)(p.block_table + (int64_t)b * p.max_pages);

    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    char *tile0 = lds_raw + wave * (kStages * kTileBytes);
    char *tile1 = tile0 + kTileBytes;

    for (int part = first_part; part < n_parts; part += stride) {
    const int t0 = p.partition_tokens > 0 ? part * p.partition_tokens : 0;
    const int t1 = p.partition_tokens > 0 ? min(L, t0 + p.partition_tokens) : L;
    const int pg_end = (t1 + kPageSize - 1) / kPageSize;
    WaveState st;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        st.o[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    st.m = kNegBig;
    st.l = 0.f;

    // Two page buffers used alternately (K tile in LDS + V rows in registers),
    // so that the loads of page n+1 are in flight while page n is consumed.  A
    // wave always issues the next load group, even past its last page (then with a
    // descriptor of zero bytes: the loads return zeros and fetch nothing), which
    // keeps the number of loads in flight fixed: "all but the newest eight" is
    // always the page to consume.
    // Page ids are fetched two pages ahead.
    int pg = t0 / kPageSize + wave;
    if (pg < pg_end) {
        PageRegs A, B;
        u32x4 ka[4];
        const int last = pg + (pg_end - 1 - pg) / kWaves * kWaves; // this wave's last page
        const int sh = p.page_shift; // a cache page is 1 << sh tiles of 16 tokens
#define ADR_TILE(T) pool_tile_checked(bt[(T) >> sh], (T), p.num_pages, sh, p.bounds, b)
        int page = ADR_TILE(pg);
        int page_next = ADR_TILE(min(pg + kWaves, last));
        load_page(A, tile0, page_rsrc(kc, page, page_bytes), page_rsrc(vc, page, page_bytes), k_lane,
                  v_lane, tok_bytes);
        for (;;) {
            page = page_next;
            page_next = ADR_TILE(min(pg + 2 * kWaves, last));
            const uint32_t range_b = pg + kWaves <= last ? page_bytes : 0u;
            load_page(B, tile1, page_rsrc(kc, page, page_bytes, range_b), page_rsrc(vc, page, page_bytes, range_b),
                      k_lane, v_lane, tok_bytes);
            wait_older_page();
            read_k_operand(ka, tile0, k_read);
            attend_page(st, A, ka, qb, p.scale_log2e, 1.f, pg * kPageSize + 4 * j, t1, j);
            pg += kWaves;
            if (pg >= pg_end)
                break;
            page = page_next;
            page_next = ADR_TILE(min(pg + 2 * kWaves, last));
            const uint32_t range_a = pg + kWaves <= last ? page_bytes : 0u;
            load_page(A, tile0, page_rsrc(kc, page, page_bytes, range_a), page_rsrc(vc, page, page_bytes, range_a),
                      k_lane, v_lane, tok_bytes);
            wait_older_page();
            read_k_operand(ka, tile1, k_read);
            attend_page(st, B, ka, qb, p.scale_log2e, 1.f, pg * kPageSize + 4 * j, t1, j);
            pg += kWaves;
            if (pg >= pg_end)
                break;
        }
#undef ADR_TILE
    }
    // the K tiles are dead from here on; the same LDS now carries the per-wave results
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // denominators: sum the four lane groups
    float l = st.l;
    l = sum_across_rows(l);

    float *sm = (float *)lds_raw;     // [kWaves][G]
    float *sl = sm + kWaves * G;      // [kWaves][G]
    float *so = sl + kWaves * G;      // [kWaves][G][D]
    if (j == 0 && r < G) {
        sm[wave * G + r] = st.m;
        sl[wave * G + r] = l;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int g = 4 * j + i;
        if (g < G) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                so[(wave * G + g) * D + 8 * r + e] = st.o[e][i];
        }
    }
    __syncthreads();
    combine_waves_and_store<D>(p, sm, sl, so, G, b, kvh, part, n_parts);
    __syncthreads(); // the next partition's K tiles go where the per-wave results lie
    }
}

hipError_t launch_decode_mfma(const DecodeParams &p, int d, hipStream_t stream)
{
    if (d != D)
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)((int64_t)p.B * p.Hkv * grid_stride(p.max_parts)));
    size_t lds = (size_t)kWaves * p.G * (D + 2) * sizeof(float); // per-wave results
    if (lds < (size_t)kWaves * kStages * kTileBytes)
        lds = (size_t)kWaves * kStages * kTileBytes;             // K tiles
    decode_mfma_kernel<<<grid, kThreads, lds, stream>>>(p);
    return hipGetLastError();
}

bool decode_mfma_supports(int d, int G) { return d == D && G >= 1 && G <= 16; }

} // namespace adr
