// Persistent matrix-core decode attention (d = 128, bf16 or fp8-e4m3 cache, G <= 16,
// B <= 512).
//
// The grid is a fixed number of workgroups (a couple per compute unit) that
// stay resident and pull work items from a ticket counter until none is left.
// An item is one (request, partition, kv-head); the four waves of a workgroup
// share it, wave w streaming pages w, w+4, ... of the partition, exactly as in
// decode_mfma.hip.  What changes is everything around the page loop:
//
//  * No empty workgroups.  Every workgroup first scans seq_lens into two
//    prefix arrays in LDS (full partitions per row, ragged last partitions per
//    row); ticket t is decoded by binary search.  Tickets enumerate all full
//    partitions first and the ragged ones last, so the work that is handed out
//    at the very end is the small pieces.
//  * No pipeline drain between items.  A wave's page stream runs across item
//    boundaries: while the last page of an item is consumed, the first page of
//    the next item is already in flight, and the next item's query is loaded
//    one item ahead.  Tickets are drawn two items ahead for that reason.
//  * K and V tiles both arrive by direct-to-LDS loads into a ring of S stages per
//    wave (K rows XOR-swizzled for the operand reads, V rows natural); S - 1
//    pages are in flight while one is consumed.  One workgroup per compute
//    unit owns (almost) its whole LDS, which is what pays for the deep ring:
//    the loads in flight keep the memory pipes fed while the waves of the
//    workgroup meet at an item's end.  The ring position is a run-time value.
//    A wave whose stream has run dry (no further page in the current or the
//    next item) fills ring slots with null loads, so the number of load groups
//    in flight never changes and one wait count serves every page; null slots
//    are skipped when their turn comes.
//  * The query operand of an item is likewise staged in LDS (one 16-row tile per
//    workgroup, fetched by wave 0 one item ahead), so no load into registers is
//    ever pending inside the page loop and the compiler adds no waits there.
//  * The cross-wave combination of an item goes through a double-buffered
//    staging area, so one barrier per item is enough.
//
// fp8 cache: a page of one kv-head is half the bytes (two loads per tile instead
// of four), and two more 4-byte direct-to-LDS loads bring the page's K and V
// scales into the tail of the ring stage.  The bytes are widened to bf16 (exact)
// after the LDS read and enter the same matrix instructions; the K scale is
// folded into the score scale and the V scale into the weights.  The ring is
// deeper, since a stage is smaller.
//
// The ticket counter and a finished-workgroups counter live in a small pool of
// static device words that are zero whenever no launch is using them: the last
// workgroup to finish puts both back to zero.
#include "mfma_page.h"

#include <algorithm>
#include <atomic>

namespace adr {

constexpr int kMaxStreamB = 512;
constexpr int kTicketSlots = 64;

// Geometry of one ring stage: K tile, V tile, then (fp8) the two scales, each
// in a 256-byte slot of its own (a 4-byte direct-to-LDS load covers 64 x 4 bytes).
template <bool FP8> struct Geo {
    static constexpr int kRow = FP8 ? D : 2 * D;          // bytes of one token of one kv-head
    static constexpr int kTile = kPageSize * kRow;        // 2 KB / 4 KB
    static constexpr int kTileLoads = kTile / 1024;       // 16-byte-per-lane loads per tile
    static constexpr int kScaleSlot = 256;
    static constexpr int kStage = 2 * kTile + (FP8 ? 2 * kScaleSlot : 0);
    static constexpr int kGroup = 2 * kTileLoads + (FP8 ? 2 : 0); // loads per page
    static constexpr int kMaxStages = FP8 ? 6 : 4;
};

__device__ uint32_t g_tickets[kTicketSlots][2];

struct StreamParams {
    DecodeParams d;
    uint32_t *ticket; // {next ticket, workgroups finished}
    int pt;           // tokens per partition (2^30 when the pass is not split)
    int stages;       // ring stages per wave (2 .. Geo::kMaxStages)
};

struct Item {
    int valid;
    int b, kvh, part;
    int t1;      // end of the token range (exclusive); the range starts at part * pt
    int n_parts; // partitions of the row (1: write the final result directly)
    int pg;      // first page of this wave
    int pg_end;  // one past the last page of the item
};

typedef const __attribute__((address_space(4))) int32_t *table_ptr;

constexpr int kMaxLdsBytes = 160 * 1024;  // LDS of one compute unit
constexpr int kQTileBytes = 16 * D * 2; // sixteen query rows (heads of a group, zero beyond G)

// LDS layout: the ring (kWaves * stages * Geo::kStage), this block, then the
// staging area float[2][kWaves][G][D] for the per-wave results of an item.
struct Shared {
    char qtile[2][kQTileBytes]; // query tile of the current / the next item, rows swizzled like K
    float ml[2][kWaves][16][2]; // per item parity, per wave: running max, denominator of each head
    int slot[2];                // tickets of the items after the current one
    int wave_tot[2][kWaves];
    int total[2];
    int pref_full[kMaxStreamB + 1];
    int pref_rag[kMaxStreamB + 1];
    int len[kMaxStreamB];
};

// largest b with pref[b] <= u  (pref is an exclusive prefix sum of length B+1)
__device__ __forceinline__ int find_row(const int *pref, int B, int u)
{
    int lo = 0, hi = B; // invariant: pref[lo] <= u < pref[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (__builtin_amdgcn_readfirstlane(pref[mid]) <= u)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

__device__ __forceinline__ Item decode_ticket(const Shared &sh, const StreamParams &sp, int ticket,
                                              int wave)
{
    Item it;
    const int Hkv = sp.d.Hkv, B = sp.d.B;
    // everything below is the same in all lanes; say so, to keep it in scalar registers
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    const int total_full = __builtin_amdgcn_readfirstlane(sh.total[0]);
    const int total_rag = __builtin_amdgcn_readfirstlane(sh.total[1]);
    it.valid = (unsigned)ticket < (unsigned)((total_full + total_rag) * Hkv);
    it.b = it.kvh = it.part = it.t1 = it.pg = it.pg_end = 0;
    it.n_parts = 1;
    if (it.valid) {
        const int unit = ticket / Hkv;
        it.kvh = ticket - unit * Hkv;
        int b, t1;
        if (unit < total_full) {
            b = find_row(sh.pref_full, B, unit);
            it.part = unit - sh.pref_full[b];
            t1 = (it.part + 1) * sp.pt;
        } else {
            b = find_row(sh.pref_rag, B, unit - total_full);
            it.part = sh.pref_full[b + 1] - sh.pref_full[b];
            t1 = sh.len[b];
        }
        const int L = sh.len[b];
        it.b = __builtin_amdgcn_readfirstlane(b);
        it.part = __builtin_amdgcn_readfirstlane(it.part);
        it.kvh = __builtin_amdgcn_readfirstlane(it.kvh);
        it.t1 = __builtin_amdgcn_readfirstlane(t1);
        const int np = L > 0 ? (L - 1) / sp.pt + 1 : 1;
        it.n_parts = __builtin_amdgcn_readfirstlane(np);
        // part * pt cannot overflow: when the pass is not split, part is 0
        it.pg = it.part * (sp.pt / kPageSize) + wave;
        it.pg_end = (it.t1 + kPageSize - 1) / kPageSize;
    }
    return it;
}

// Fetch the query tile of one item into LDS (one wave calls this): sixteen rows
// of 256 bytes, row t stored with its chunks XOR-permuted by t exactly like a K
// tile.  The descriptor spans the G rows of the group; rows beyond it are out of
// range (their content is never used: they only feed score columns >= G).
__device__ __forceinline__ void issue_query(char *qtile, const StreamParams &sp, const Item &it,
                                            const uint32_t (&q_lane)[4])
{
    const char *base = (const char *)(sp.d.q + (int64_t)it.b * sp.d.q_row_stride +
                                      (int64_t)it.kvh * sp.d.G * D);
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, it.valid ? sp.d.G * D * 2 : 0, 0x00020000);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rs, (__attribute__((address_space(3))) void *)(qtile + i * 1024), 16, q_lane[i], 0, 0, 0);
    asm volatile("" ::: "memory");
}

// The direct-to-LDS loads of one page for one kv-head into ring stage `tile`:
// K rows (swizzled), V rows (natural) and, for an fp8 cache, the page's two
// scales (lane 0 only: the other lanes' offsets are out of the descriptor's range).
template <bool FP8>
__device__ __forceinline__ void issue_page(char *tile, __amdgpu_buffer_rsrc_t krsrc,
                                           __amdgpu_buffer_rsrc_t vrsrc, __amdgpu_buffer_rsrc_t ksrsrc,
                                           __amdgpu_buffer_rsrc_t vsrsrc, const uint32_t (&k_lane)[4],
                                           const uint32_t (&v_lane)[4], uint32_t s_lane,
                                           uint32_t head_bytes, uint32_t scale_bytes)
{
    typedef Geo<FP8> geo;
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < geo::kTileLoads; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            krsrc, (__attribute__((address_space(3))) void *)(tile + i * 1024), 16, k_lane[i],
            head_bytes, 0, kStreamOnce);
#pragma unroll
    for (int i = 0; i < geo::kTileLoads; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            vrsrc, (__attribute__((address_space(3))) void *)(tile + geo::kTile + i * 1024), 16,
            v_lane[i], head_bytes, 0, kStreamOnce);
    if (FP8) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            ksrsrc, (__attribute__((address_space(3))) void *)(tile + 2 * geo::kTile), 4, s_lane,
            scale_bytes, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            vsrsrc, (__attribute__((address_space(3))) void *)(tile + 2 * geo::kTile + geo::kScaleSlot),
            4, s_lane, scale_bytes, 0, 0);
    }
    asm volatile("" ::: "memory");
}

// Workgroup barrier for the item loop: orders this wave's LDS accesses (they
// complete in issue order once the LDS counter has drained) without waiting for
// the direct-to-LDS page loads still in flight, which target ring stages that
// no other wave ever touches.
__device__ __forceinline__ void ring_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Wait until all but the newest S - 1 load groups have landed.
template <bool FP8>
__device__ __forceinline__ void wait_ring(int stages)
{
#define ADR_WAIT_CASE(S)                                                                          \
    case S:                                                                                       \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 1) * Geo<FP8>::kGroup) : "memory");          \
        break;
    switch (stages) {
        ADR_WAIT_CASE(6)
        ADR_WAIT_CASE(5)
        ADR_WAIT_CASE(4)
        ADR_WAIT_CASE(3)
    default:
        ADR_WAIT_CASE(2)
    }
#undef ADR_WAIT_CASE
}

template <bool FP8>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 2)))
void decode_stream_kernel(const StreamParams sp)
{
    const DecodeParams &p = sp.d;
    typedef Geo<FP8> geo;
    constexpr int kStageBytes = geo::kStage;
    const int S = sp.stages;
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const int ring_bytes = kWaves * S * kStageBytes;
    Shared &sh = *(Shared *)(lds_raw + ring_bytes);
    float *staging = (float *)(lds_raw + ring_bytes + sizeof(Shared)); // [2][kWaves][G][D]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15;
    const int j = lane >> 4;
    const int B = p.B, Hkv = p.Hkv, G = p.G;

    // ---- partitions per row: exclusive prefix sums over the rows, four rows per thread
    {
        int f[4], g[4], sf = 0, sg = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = tid * 4 + i;
            int L = 0;
            f[i] = g[i] = 0;
            if (row < B) {
                L = max(min(p.seq_lens[row], p.max_seq_len), 0);
                sh.len[row] = L;
                f[i] = L / sp.pt;
                g[i] = (L % sp.pt != 0 || L == 0) ? 1 : 0; // an empty row still owns one (empty) item
            }
            sf += f[i];
            sg += g[i];
        }
        int xf = sf, xg = sg; // inclusive scan over the lanes of the wave
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int yf = __shfl_up(xf, off), yg = __shfl_up(xg, off);
            if (lane >= off) {
                xf += yf;
                xg += yg;
            }
        }
        if (lane == 63) {
            sh.wave_tot[0][wave] = xf;
            sh.wave_tot[1][wave] = xg;
        }
        __syncthreads();
        int bf = 0, bg = 0, tf = 0, tg = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (w < wave) {
                bf += sh.wave_tot[0][w];
                bg += sh.wave_tot[1][w];
            }
            tf += sh.wave_tot[0][w];
            tg += sh.wave_tot[1][w];
        }
        int ef = bf + xf - sf, eg = bg + xg - sg;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = tid * 4 + i;
            if (row < B) {
                sh.pref_full[row] = ef;
                sh.pref_rag[row] = eg;
            }
            ef += f[i];
            eg += g[i];
        }
        if (tid == 0) {
            sh.pref_full[B] = tf;
            sh.pref_rag[B] = tg;
            sh.total[0] = tf;
            sh.total[1] = tg;
            sh.slot[0] = (int)atomicAdd(sp.ticket, 1u);
            sh.slot[1] = (int)atomicAdd(sp.ticket, 1u);
        }
        __syncthreads();
    }

    // ---- per-lane constants
    // bf16: a row is sixteen 16-byte chunks and a load covers four rows; slot c of row t
    //       holds chunk c ^ t.  Step kk of QK^T reads chunk kk*4 + j of row r (8 elements).
    // fp8:  a row is eight 16-byte chunks and a load covers eight rows; slot c of row t
    //       holds chunk c ^ (t & 7).  The same 8 elements are the 8-byte piece kk*4 + j.
    const uint32_t tok_bytes = (uint32_t)Hkv * geo::kRow;
    const uint32_t page_bytes = kPageSize * tok_bytes;
    uint32_t k_lane[4], v_lane[4], q_lane[4], k_read[4], q_read[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = 4 * i + j; // query-tile row this lane fetches in load i
        q_lane[i] = t * (D * 2) + ((r ^ t) * 16);
        q_read[i] = r * (D * 2) + (((i * 4 + j) ^ r) * 16);
        if (FP8) {
            const int tf = 8 * (i & 1) + (lane >> 3), c = lane & 7; // row / slot of load i (i < 2)
            k_lane[i] = tf * tok_bytes + ((c ^ (tf & 7)) * 16);
            v_lane[i] = tf * tok_bytes + c * 16;
            const int piece = i * 4 + j;
            k_read[i] = r * D + (((piece >> 1) ^ (r & 7)) * 16) + (piece & 1) * 8;
        } else {
            k_lane[i] = t * tok_bytes + ((r ^ t) * 16);
            v_lane[i] = t * tok_bytes + r * 16;
            k_read[i] = q_read[i];
        }
    }
    // V operand: rows 4j + u, the 8 elements 8r .. 8r+7
    const uint32_t v_read = (4 * j) * geo::kRow + r * (geo::kRow / 16);
    const uint32_t s_lane = lane == 0 ? 0u : 0x7ffffff0u; // scale loads: only lane 0 is in range
    const char *kc = (const char *)p.k_cache;
    const char *vc = (const char *)p.v_cache;
    char *ring = lds_raw + wave * (S * kStageBytes);
    const __amdgpu_buffer_rsrc_t null_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)kc, 0, 0, 0x00020000); // every read is out of range: zeros
    const int scale_range = FP8 ? p.num_pages * Hkv * 4 : 0;
    const __amdgpu_buffer_rsrc_t ks_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)(FP8 ? (const void *)p.k_scale : (const void *)kc), 0, scale_range, 0x00020000);
    const __amdgpu_buffer_rsrc_t vs_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)(FP8 ? (const void *)p.v_scale : (const void *)kc), 0, scale_range, 0x00020000);

    Item C = decode_ticket(sh, sp, sh.slot[0], wave);
    Item N = decode_ticket(sh, sp, sh.slot[1], wave);
    if (wave == 0) {
        issue_query(sh.qtile[0], sp, C, q_lane);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();

    // ---- load cursor: the next page of this wave's stream to be issued.  It runs
    // through the current item and on into the next one, never further.  It keeps
    // its own copy of what it needs from the item it is in.
    int ld_in_next = 0;
    int ld_pg = C.pg, ld_end = C.valid ? C.pg_end : 0;
    uint32_t ld_head = (uint32_t)C.kvh * geo::kRow;
    int ld_kvh = C.kvh;
    table_ptr ld_bt = (table_ptr)(p.block_table + (int64_t)C.b * p.max_pages);
    int ld_ok = 0, ld_id = 0;
#define ADR_SETTLE()                                                                              \
    do { /* move the cursor to the next existing page and fetch its page id */                    \
        if (!ld_in_next && ld_pg >= ld_end) {                                                     \
            ld_in_next = 1;                                                                       \
            ld_pg = N.pg;                                                                         \
            ld_end = N.valid ? N.pg_end : 0;                                                      \
            ld_head = (uint32_t)N.kvh * geo::kRow;                                                \
            ld_kvh = N.kvh;                                                                       \
            ld_bt = (table_ptr)(p.block_table + (int64_t)N.b * p.max_pages);                      \
        }                                                                                         \
        ld_ok = ld_pg < ld_end;                                                                   \
        if (ld_ok)                                                                                \
            ld_id = clamp_page(ld_bt[ld_pg], p.num_pages);                                        \
    } while (0)
#define ADR_ISSUE(STAGE)                                                                          \
    do { /* fill a ring stage with the cursor's page, or with a group of null loads */            \
        const int stage_ = (STAGE);                                                               \
        char *tile_ = ring + stage_ * kStageBytes;                                                \
        if (ld_ok) {                                                                              \
            issue_page<FP8>(tile_, page_rsrc(kc, ld_id, page_bytes),                              \
                            page_rsrc(vc, ld_id, page_bytes), ks_rsrc, vs_rsrc, k_lane, v_lane,   \
                            s_lane, ld_head, (uint32_t)(ld_id * Hkv + ld_kvh) * 4u);              \
            real_mask |= 1 << stage_;                                                             \
            ld_pg += kWaves;                                                                      \
            ADR_SETTLE();                                                                         \
        } else {                                                                                  \
            issue_page<FP8>(tile_, null_rsrc, null_rsrc, null_rsrc, null_rsrc, k_lane, v_lane,    \
                            s_lane, 0, 0);                                                        \
            real_mask &= ~(1 << stage_);                                                          \
        }                                                                                         \
    } while (0)
    ADR_SETTLE();
    // Ring state: stages stage .. stage+S-2 (mod S) hold the next S-1 slots of the
    // stream in order, stage-1 is free; real_mask marks the slots that hold a page.
    int stage = 0, real_mask = 0;
    for (int s0 = 0; s0 < S - 1; ++s0)
        ADR_ISSUE(s0);

    uint32_t next_ticket = 0;
    // Drawn once per item, after the item's first page has been consumed (so that
    // nothing at the top of an item waits for these round trips): the ticket of the
    // item after N, and N's query.  The counter's address may reach its scalar
    // registers through a vector-lane read just before the statement; the five
    // wait states such a value needs before a memory instruction may use it are
    // not inserted around hand-written instructions, hence the s_nop.
#define ADR_LOOK_AHEAD()                                                                          \
    do {                                                                                          \
        if (tid == 0)                                                                             \
            asm volatile("s_nop 4\n\tglobal_atomic_add %0, %1, %2, %3 sc0"                        \
                         : "=&v"(next_ticket)                                                     \
                         : "v"(0), "v"(1), "s"(sp.ticket)                                         \
                         : "memory");                                                             \
        if (wave == 0)                                                                            \
            issue_query(sh.qtile[(k + 1) & 1], sp, N, q_lane);                                    \
    } while (0)

    for (int k = 0; C.valid; ++k) {
        WaveState st;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            st.o[e] = f32x4{0.f, 0.f, 0.f, 0.f};
        st.m = kNegBig;
        st.l = 0.f;
        u32x4 qb[4]; // B operand of QK^T: head r's query, chunk order matching the K reads
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            qb[kk] = *(const u32x4 *)(sh.qtile[k & 1] + q_read[kk]);

        bool looked = false;
        for (int pg = C.pg; pg < C.pg_end; pg += kWaves) {
            // Step through the ring to the slot that holds this page: every step
            // refills the stage freed by the step before; null slots are passed over.
            for (;;) {
                ADR_ISSUE(stage == 0 ? S - 1 : stage - 1);
                if ((real_mask >> stage) & 1)
                    break;
                stage = stage + 1 == S ? 0 : stage + 1;
            }
            wait_ring<FP8>(S);
            const char *tile = ring + stage * kStageBytes;
            PageRegs pr;
            u32x4 ka[4];
            float score_scale = p.scale_log2e, p_scale = 1.f;
            if (FP8) {
                u32x2 vraw[4], kraw[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    vraw[u] = *(const u32x2 *)(tile + geo::kTile + v_read + u * geo::kRow);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    kraw[kk] = *(const u32x2 *)(tile + k_read[kk]);
                score_scale *= *(const float *)(tile + 2 * geo::kTile);
                p_scale = *(const float *)(tile + 2 * geo::kTile + geo::kScaleSlot);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    pr.v[u] = fp8x8_to_bf16x8(vraw[u]);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    ka[kk] = fp8x8_to_bf16x8(kraw[kk]);
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    pr.v[u] = *(const u32x4 *)(tile + geo::kTile + v_read + u * geo::kRow);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    ka[kk] = *(const u32x4 *)(tile + k_read[kk]);
            }
            attend_page(st, pr, ka, qb, score_scale, p_scale, pg * kPageSize + 4 * j, C.t1, j);
            real_mask &= ~(1 << stage);
            stage = stage + 1 == S ? 0 : stage + 1;
            if (!looked) {
                looked = true;
                ADR_LOOK_AHEAD();
            }
        }
        if (!looked)
            ADR_LOOK_AHEAD();

        // ---- combine the four waves through the staging area of this item's parity
        float l = st.l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        // Wave 0 needs the ticket it drew and the query tile it requested after the
        // item's first page.  Each later page of the wave issued one more load
        // group, so after S - 1 of them the ring's own wait count covers both;
        // a shorter item waits for everything.
        if (wave == 0) {
            if (C.pg + (S - 1) * kWaves < C.pg_end)
                wait_ring<FP8>(S);
            else
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        float *so = staging + ((k & 1) * kWaves + wave) * (G * D); // [G][D]
        if (j == 0 && r < G) {
            sh.ml[k & 1][wave][r][0] = st.m;
            sh.ml[k & 1][wave][r][1] = l;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int g = 4 * j + i;
            if (g < G) {
                *(f32x4 *)(so + g * D + 8 * r) = f32x4{st.o[0][i], st.o[1][i], st.o[2][i], st.o[3][i]};
                *(f32x4 *)(so + g * D + 8 * r + 4) = f32x4{st.o[4][i], st.o[5][i], st.o[6][i], st.o[7][i]};
            }
        }
        if (tid == 0)
            sh.slot[k & 1] = (int)next_ticket;
        ring_barrier();
        // Nothing written above is written again before the barrier of the item after
        // the next one, which no wave reaches before all have finished reading here.

        const float *sbase = staging + (k & 1) * kWaves * (G * D);
        for (int idx = tid; idx < G * D; idx += kThreads) {
            const int g = idx / D, dd = idx - g * D;
            float M = sh.ml[k & 1][0][g][0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w)
                M = fmaxf(M, sh.ml[k & 1][w][g][0]);
            float acc = 0.f, den = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float f = fast_exp2(sh.ml[k & 1][w][g][0] - M);
                acc += f * sbase[w * (G * D) + g * D + dd];
                den += f * sh.ml[k & 1][w][g][1];
            }
            const float o = den > 0.f ? acc / den : 0.f;
            const float lse = den > 0.f ? (M + fast_log2(den)) * kLn2 : -INFINITY;
            const int h = C.kvh * G + g;
            if (C.n_parts == 1) {
                const int64_t off = ((int64_t)C.b * p.Hq + h) * D + dd;
                if (p.out_f32)
                    ((float *)p.out)[off] = o;
                else
                    ((uint16_t *)p.out)[off] = (uint16_t)f32_to_bf16(o);
                if (p.lse && dd == 0)
                    p.lse[(int64_t)C.b * p.Hq + h] = lse;
            } else {
                const int64_t row = ((int64_t)C.b * p.max_parts + C.part) * p.Hq + h;
                p.part_o[row * D + dd] = o;
                if (dd == 0)
                    p.part_lse[row] = lse;
            }
        }
        const int following = sh.slot[k & 1];

        // ---- next item becomes current
        C = N;
        N = decode_ticket(sh, sp, following, wave);
        // The cursor is always inside the item that has just become current (issuing
        // the last page of an item moves it on, and so does an item without pages).
        ld_in_next = 0;
        if (!ld_ok)
            ADR_SETTLE(); // it had run out of pages there: move on into the new next item
    }

#undef ADR_LOOK_AHEAD
#undef ADR_ISSUE
#undef ADR_SETTLE

    // ---- hand the counters back to zero once every workgroup is through
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (tid == 0) {
        const uint32_t done = atomicAdd(sp.ticket + 1, 1u);
        if (done == gridDim.x - 1) {
            atomicExch(sp.ticket, 0u);
            atomicExch(sp.ticket + 1, 0u);
        }
    }
}

namespace {
std::atomic<unsigned> g_next_slot{0};
}

constexpr bool kStreamKernelEnabled = true;

bool decode_stream_supports(int d, int G, int B)
{
    return kStreamKernelEnabled && d == D && G >= 1 && G <= 16 && B <= kMaxStreamB;
}

hipError_t launch_decode_stream(const DecodeParams &p, int d, bool fp8, hipStream_t stream)
{
    if (!decode_stream_supports(d, p.G, p.B))
        return hipErrorInvalidValue;
    // per-device set-up, once: address of the counter pool, LDS limit, grid size
    struct DeviceInfo {
        uint32_t *tickets = nullptr;
        int workgroups = 0;
    };
    static DeviceInfo info[64];
    static std::atomic<int> ready[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    // Ring depth: what one workgroup's LDS holds next to the staging area of the group size.
    const size_t fixed = sizeof(Shared) + (size_t)2 * kWaves * p.G * D * sizeof(float);
    const int stage_bytes = fp8 ? Geo<true>::kStage : Geo<false>::kStage;
    int stages = (int)(((size_t)kMaxLdsBytes - fixed) / ((size_t)kWaves * stage_bytes));
    stages = std::min(stages, fp8 ? Geo<true>::kMaxStages : Geo<false>::kMaxStages);
    if (stages < 2)
        return hipErrorInvalidValue;
    const size_t lds = (size_t)kWaves * stages * stage_bytes + fixed;
    if (!ready[dev].load(std::memory_order_acquire)) {
        DeviceInfo di;
        if ((e = hipGetSymbolAddress((void **)&di.tickets, HIP_SYMBOL(g_tickets))) != hipSuccess)
            return e;
        if ((e = hipFuncSetAttribute((const void *)decode_stream_kernel<false>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes)) != hipSuccess)
            return e;
        if ((e = hipFuncSetAttribute((const void *)decode_stream_kernel<true>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes)) != hipSuccess)
            return e;
        int cus = 0;
        if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess)
            return e;
        di.workgroups = cus; // one workgroup per compute unit: each takes most of its LDS
        info[dev] = di;
        ready[dev].store(1, std::memory_order_release);
    }
    StreamParams sp;
    sp.d = p;
    sp.ticket = info[dev].tickets + 2 * (g_next_slot.fetch_add(1) % kTicketSlots);
    sp.pt = p.partition_tokens > 0 ? p.partition_tokens : (1 << 30);
    sp.stages = stages;
    int64_t grid = (int64_t)p.B * p.Hkv * p.max_parts;
    if (grid > info[dev].workgroups)
        grid = info[dev].workgroups;
    if (fp8)
        decode_stream_kernel<true><<<dim3((unsigned)grid), kThreads, lds, stream>>>(sp);
    else
        decode_stream_kernel<false><<<dim3((unsigned)grid), kThreads, lds, stream>>>(sp);
    return hipGetLastError();
}

} // namespace adr
