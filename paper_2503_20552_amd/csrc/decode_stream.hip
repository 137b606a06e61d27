// Persistent matrix-core decode attention (d = 128, bf16 or fp8-e4m3 cache, G <= 16,
// B <= 512).
//
// The grid is one workgroup of four waves per compute unit (two for an fp8 cache
// when they fit: see the launch function).  The workgroups stay
// resident and pull work items from a ticket counter until none is left.  An
// item is one (request, partition, kv-head); the four waves share it, wave w
// taking pages w, w+4, ... of the partition.  Apart from that shared result the
// waves run on their own: there is no barrier in the item loop.
//
//  * No empty workgroups.  Every workgroup first scans seq_lens into two prefix
//    arrays in LDS (full partitions per row, ragged last partitions per row);
//    ticket t is decoded by binary search.  Tickets enumerate all full
//    partitions first and the ragged ones last, so the work handed out at the
//    very end is the small pieces.  When a pass has tens of thousands of
//    partitions, an item is a run of two or four neighbouring partitions of a
//    row: what an item costs besides its pages (records, staging, combining) is
//    paid that much less often.
//  * Items are announced through a small queue of records in LDS.  The ticket of
//    item k+3 is drawn at the start of item k by wave k mod 4, which decodes and
//    publishes it when it has finished its share of item k; every wave picks a
//    record up one item before it becomes its "next" item.  A record's sequence
//    stamp is written last; readers poll it.
//  * A wave's page stream runs across item boundaries.  K and V tiles arrive by
//    direct-to-LDS loads into a ring of S stages per wave (K rows XOR-swizzled
//    for the operand reads, V rows natural).  The ring is kept full; a wave
//    whose stream has run dry fills slots with null loads, so the number of load
//    groups in flight is always known and plain wait counts serve every page.
//    Null slots are passed over when they reach the head of the ring.
//  * Pages are consumed two at a time when the wave's next two pages are both in
//    the ring: one softmax step over 32 tokens, and P V as 16x16x32 products.
//  * Each wave fetches the query rows of its next item into a tile of its own
//    (direct-to-LDS as well, one item ahead), so no load into registers is ever
//    pending inside the page loop and the compiler adds no waits there.
//  * The per-wave results of an item meet in a staging buffer (two buffers,
//    used alternately).  Each wave adds itself to the buffer's arrival counter;
//    the waves take turns to combine, one item late: at the end of item k the
//    wave whose turn it is combines item k - 1 out of the other buffer (checking
//    that its counter has reached four, which it almost always has), writes the
//    output and hands that buffer back.  Nobody falls in step with the slowest
//    wave.  (Leaving the combine to the last wave to arrive would load every
//    item's extra work on the wave the others are already waiting for.)
//
// fp8 cache: a page of one kv-head is half the bytes (two loads per tile instead
// of four), and two more 4-byte direct-to-LDS loads bring the page's K and V
// scales into the tail of the ring stage.  The bytes are widened to bf16 (exact)
// after the LDS read and enter the same matrix instructions; the K scale is
// folded into the score scale and the V scale into the weights.
//
// Every wait on another wave is bounded: a wave that has polled an LDS word for
// far longer than any legitimate delay counts a fault -- in the launch's control
// block, in the call's status word and in a device-wide counter (readable through
// adr_stream_fault_count) -- and carries on, so the grid always drains.  From then
// on its workgroup stores NaN instead of results, and the last workgroup of the
// launch to finish overwrites the launch's rows of out / lse (and the partitions'
// lse) with NaN: a row that a broken hand-shake left stale or wrong cannot pass as
// a result.  (A split pass's merge reads the status word and does the same.)
//
// The ticket counter and a finished-workgroups counter live in the launch's control
// block: in the caller's workspace when there is one, else in a small pool of static
// device words.  They are zero whenever no launch is using them: the last workgroup
// to finish puts them back to zero.
#include "mfma_page.h"

#include <algorithm>
#include <atomic>

namespace adr {

constexpr int kMaxStreamB = 512;
constexpr int kTicketSlots = 256; // counter pairs: the lower half serves direct launches, the upper half recorded ones
constexpr int kQueue = 8;          // item records kept in LDS (power of two)
// polls of an LDS word before a wait is declared failed: DecodeParams::spin_limit, kSpinLimit by default
// (seconds: an unsplit row of millions of tokens keeps a wave busy for tens of ms)
constexpr int kSpinLimitAfterFault = 64; // ... once a wait of this workgroup has failed
constexpr int kCoalesceItems = 8192;     // items (of the caller's partition size) per doubling of the item size:
                                         // measured neutral below about 16K items, -5 to -10 % at 40K

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

// Launch control blocks for calls without a workspace, and the status word such calls share.
__device__ uint32_t g_pool[kTicketSlots][4];
__device__ uint32_t g_pool_status[kControlBlockWords];
__device__ unsigned long long g_stream_faults;

struct StreamParams {
    DecodeParams d;
    uint32_t *ctl;    // the launch's control block: kLaunchTicket, kLaunchFinished, kLaunchExpired
    uint32_t *status; // the call's status block
    unsigned long long *faults;
    int pt;           // tokens per partition (2^30 when the pass is not split)
    int stages;       // ring stages per wave (2 .. Geo::kMaxStages)
    int nb;           // staging buffers (1 or 2)
    int q_rows;       // rows of a wave's query tile (G rounded up to 4)
};

// One work item as the queue carries it (all fields wave-uniform).
struct Item {
    int valid;
    int b, kvh, part;
    int t1;      // end of the token range (exclusive); the range starts at part * pt
    int n_parts; // partitions of the row (1: write the final result directly)
};

struct alignas(16) Rec {
    int seq; // index of the item this record describes; written last
    int valid, b, kvh, part, t1, n_parts, pad;
};

typedef const __attribute__((address_space(4))) int32_t *table_ptr;

constexpr int kMaxLdsBytes = 160 * 1024; // LDS of one compute unit

// LDS layout: the ring (kWaves * stages * Geo::kStage), the query tiles
// (kWaves * q_rows * 256 bytes: one per wave, refilled with the next item's rows as soon as an
// item's rows have been read out), this block, then the staging area
// float[nb][kWaves][G][D] for the per-wave results of an item.
struct alignas(16) Shared {
    Rec rec[kQueue];
    int gen[2];    // per staging buffer: how many items have been combined out of it
    int arrive[2]; // per staging buffer: waves that have delivered the current item
    int first[3];  // tickets of the first three items
    int failed;    // a bounded wait of this workgroup has expired
    float ml[2][kWaves][16][2]; // per staging buffer, per wave: running max, denominator of each head
    int wave_tot[2][kWaves];
    int total[2];
    int pref_full[kMaxStreamB + 1];
    int pref_rag[kMaxStreamB + 1];
};

// largest b < B with pref[b] <= u  (pref is an exclusive prefix sum, pref[0] = 0 <= u; B <= 512);
// *at_row receives pref[b].
// Called by a whole wave: sixty-four lanes probe every eighth entry, eight lanes the eight
// entries of the block found, and the counts of the two ballots give the row -- two LDS round
// trips instead of the nine of a binary search (each costs the wave a few hundred cycles).
__device__ __forceinline__ int find_row(const int *pref, int B, int u, int *at_row)
{
    const int lane = threadIdx.x & 63;
    const int coarse = lane * 8;
    const bool below = coarse < B && pref[coarse] <= u;
    const int block = __popcll(__ballot(below)) - 1;
    const int fine = block * 8 + (lane & 7);
    const int value = lane < 8 && fine < B ? pref[fine] : 0x7fffffff;
    const int hits = __popcll(__ballot(value <= u));
    *at_row = __builtin_amdgcn_readlane(value, hits - 1);
    return block * 8 + hits - 1;
}

// A row's length as the scan in the kernel's set-up took it (the row index is the same in all lanes:
// a scalar load).
__device__ __forceinline__ int row_length(const StreamParams &sp, int b)
{
    // (read through the constant address space: a scalar load, which no load of the ring waits behind)
    const int L = ((const __attribute__((address_space(4))) int32_t *)sp.d.seq_lens)[__builtin_amdgcn_readfirstlane(b)];
    return max(min(L, sp.d.max_seq_len), 0);
}

// cshift: tickets enumerate runs of 1 << cshift partitions (see the kernel's set-up); it.part
// counts such runs, it.n_parts stays the row's number of partitions as the caller defined them.
// total_full / total_rag: the item counts the scan left in sh.total, kept in registers.
__device__ __forceinline__ Item decode_ticket(const Shared &sh, const StreamParams &sp, int ticket, int cshift,
                                              int total_full, int total_rag)
{
    Item it;
    const int Hkv = sp.d.Hkv, B = sp.d.B;
    const int pt = sp.pt << cshift;
    // everything below is the same in all lanes; say so, to keep it in scalar registers
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    it.valid = (unsigned)ticket < (unsigned)((total_full + total_rag) * Hkv);
    it.b = it.kvh = it.part = it.t1 = 0;
    it.n_parts = 1;
    if (it.valid) {
        const int unit = ticket / Hkv;
        it.kvh = ticket - unit * Hkv;
        int b, at_row, L, t1;
        if (unit < total_full) {
            b = find_row(sh.pref_full, B, unit, &at_row);
            L = row_length(sp, b);
            it.part = unit - at_row;
            t1 = (it.part + 1) * pt;
        } else {
            b = find_row(sh.pref_rag, B, unit - total_full, &at_row);
            L = row_length(sp, b);
            it.part = L / pt; // the full items of the row come before its ragged one
            t1 = L;
        }
        it.b = __builtin_amdgcn_readfirstlane(b);
        it.part = __builtin_amdgcn_readfirstlane(it.part);
        it.kvh = __builtin_amdgcn_readfirstlane(it.kvh);
        it.t1 = __builtin_amdgcn_readfirstlane(t1);
        const int np = L > 0 ? (L - 1) / sp.pt + 1 : 1;
        it.n_parts = __builtin_amdgcn_readfirstlane(np);
    }
    return it;
}

// The flags the waves exchange live in LDS, and the LDS executes one wave's
// accesses in the order they were issued.  So a flag written after the data it
// guards is seen after that data, and data read after a flag was seen is at
// least as new as the flag: nothing but the compiler has to be kept from
// reordering.  (Acquire/release atomics would also wait for the page loads in
// flight, which is exactly what the ring must not do.)
//
// The flag accesses are written as instructions by hand: the compiler would
// otherwise guard an atomic LDS access with a wait for all direct-to-LDS loads.
__device__ __forceinline__ void lds_order() { asm volatile("" ::: "memory"); }

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}

__device__ __forceinline__ int flag_read(const int *word)
{
    int v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(lds_address(word)) : "memory");
    return v;
}

__device__ __forceinline__ void flag_write(int *word, int value)
{
    asm volatile("ds_write_b32 %0, %1" ::"v"(lds_address(word)), "v"(value) : "memory");
}

// Add without waiting for anything: the LDS takes it in this wave's program order, behind
// the writes issued before it.
__device__ __forceinline__ void flag_add_async(int *word, int value)
{
    asm volatile("ds_add_u32 %0, %1" ::"v"(lds_address(word)), "v"(value) : "memory");
}

// What a wave needs to wait for another one: the workgroup's "a wait has expired" flag in LDS,
// and for how long to poll.
struct Waits {
    int *failed;
    int limit;
};

// The kernel's argument block.  Code that runs only when something has gone wrong reads what it
// needs of the parameters from here, so that none of it occupies registers through the item loop.
__device__ __forceinline__ const __attribute__((address_space(4))) StreamParams *argument_block()
{
    return (const __attribute__((address_space(4))) StreamParams *)__builtin_amdgcn_kernarg_segment_ptr();
}

// An expired wait is counted in the launch's control block, in the call's status word and
// device-wide, and flagged in the workgroup.
__device__ __forceinline__ void count_fault(const Waits &w)
{
    if ((threadIdx.x & 63) == 0) {
        flag_write(w.failed, 1);
        atomicAdd(argument_block()->faults, 1ull);
        atomicAdd(argument_block()->ctl + kLaunchExpired, 1u);
        atomicAdd(argument_block()->status + kStatusExpiredWaits, 1u);
    }
}

// Poll an LDS word until it holds `want`.  Returns false (and counts a fault)
// when it never does; the caller then goes on without what it waited for.
__device__ __forceinline__ bool poll_equal(int *word, int want, const Waits &w)
{
    int limit = w.limit;
    for (int spin = 0; spin < limit; ++spin) {
        if (__builtin_amdgcn_readfirstlane(flag_read(word)) == want) {
            lds_order();
            return true;
        }
        if (spin == 0 && __builtin_amdgcn_readfirstlane(flag_read(w.failed)))
            limit = min(limit, kSpinLimitAfterFault);
        __builtin_amdgcn_s_sleep(1);
    }
    count_fault(w);
    return false;
}

// The same, reading a second word (`also`) in the round trips of the first; *also_value
// receives what it held at the last poll (or holds now, when no poll was made).
__device__ __forceinline__ bool poll_equal_also(int *word, int want, const Waits &w, const int *also,
                                                int *also_value)
{
    int limit = w.limit, extra = 0;
    bool ok = false;
    for (int spin = 0; spin < limit && !ok; ++spin) {
        int v;
        asm volatile("ds_read_b32 %0, %2\n\tds_read_b32 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(v), "=&v"(extra)
                     : "v"(lds_address(word)), "v"(lds_address(also))
                     : "memory");
        ok = __builtin_amdgcn_readfirstlane(v) == want;
        if (!ok) {
            if (spin == 0 && __builtin_amdgcn_readfirstlane(flag_read(w.failed)))
                limit = min(limit, kSpinLimitAfterFault);
            __builtin_amdgcn_s_sleep(1);
        }
    }
    if (ok) {
        lds_order();
    } else {
        count_fault(w);
        extra = flag_read(also);
    }
    *also_value = __builtin_amdgcn_readfirstlane(extra);
    return ok;
}

__device__ __forceinline__ void publish(Rec &rec, const Item &it, int seq)
{
    if ((threadIdx.x & 63) == 0) {
        rec.valid = it.valid;
        rec.b = it.b;
        rec.kvh = it.kvh;
        rec.part = it.part;
        rec.t1 = it.t1;
        rec.n_parts = it.n_parts;
        lds_order();
        flag_write(&rec.seq, seq);
    }
}

// `also`, when given, is another LDS word read in the same round trip (every dependent LDS access
// costs a wave a few hundred cycles here); its value comes back in *also_value.
__device__ __forceinline__ Item fetch(Rec &rec, int seq, const Waits &w, const int *also = nullptr,
                                      int *also_value = nullptr)
{
    // The record is 32 bytes; its stamp is written last, so a copy whose stamp is the
    // wanted one is whole.  The common case is one round trip.
    Item it;
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    i32x4 lo, hi;
    if (also) {
        int extra;
        asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %3 offset:16\n\tds_read_b32 %2, %4\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(lo), "=&v"(hi), "=&v"(extra)
                     : "v"(lds_address(&rec)), "v"(lds_address(also))
                     : "memory");
        *also_value = __builtin_amdgcn_readfirstlane(extra);
    } else {
        asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:16\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(lo), "=&v"(hi)
                     : "v"(lds_address(&rec))
                     : "memory");
    }
    bool ok = __builtin_amdgcn_readfirstlane(lo[0]) == seq;
    if (!ok) {
        ok = poll_equal(&rec.seq, seq, w);
        asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:16\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(lo), "=&v"(hi)
                     : "v"(lds_address(&rec))
                     : "memory");
    }
    it.valid = ok ? __builtin_amdgcn_readfirstlane(lo[1]) : 0;
    it.b = __builtin_amdgcn_readfirstlane(lo[2]);
    it.kvh = __builtin_amdgcn_readfirstlane(lo[3]);
    it.part = __builtin_amdgcn_readfirstlane(hi[0]);
    it.t1 = __builtin_amdgcn_readfirstlane(hi[1]);
    it.n_parts = __builtin_amdgcn_readfirstlane(hi[2]);
    if (!ok) {
        // The record never came, and the slot holds whatever the LDS held: the wave goes on as if the
        // item were past the end, with the fields of such an item.  (The load cursor starts from the
        // item's partition whether the item is valid or not; a negative page index out of a stale
        // word would pass for a page in front of the item's end and send a scalar load, which no
        // descriptor bounds, to a wild address.)
        it.b = it.kvh = it.part = it.t1 = 0;
        it.n_parts = 1;
    }
    return it;
}

// Fetch the query rows of one item into this wave's LDS tile: rows of 256 bytes,
// row t stored with its chunks XOR-permuted by t exactly like a K tile.  The
// descriptor spans the G rows of the group; a row beyond it is out of range and
// nobody reads it.
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
        if (4 * i < sp.q_rows)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs, (__attribute__((address_space(3))) void *)(qtile + i * 1024), 16, q_lane[i], 0, 0, 0);
    asm volatile("" ::: "memory");
}

// Half of the direct-to-LDS loads of one page for one kv-head into ring stage
// `tile`: WHICH = 0 the K rows (swizzled), WHICH = 1 the V rows (natural), each
// followed, for an fp8 cache, by the page's scale of that tensor (lane 0 only: the
// other lanes' offsets are out of the descriptor's range).  The two halves of a
// page are issued separately so that a step's loads can be spread between its
// arithmetic: a wave that issues sixteen of them back to back sits in the queue
// of the compute unit's one load unit behind the other waves' loads.
template <bool FP8, int WHICH>
__device__ __forceinline__ void issue_half(char *tile, __amdgpu_buffer_rsrc_t rsrc,
                                           __amdgpu_buffer_rsrc_t scale_rsrc, const uint32_t (&lane_off)[4],
                                           uint32_t s_lane, uint32_t head_bytes, uint32_t scale_bytes)
{
    typedef Geo<FP8> geo;
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < geo::kTileLoads; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc, (__attribute__((address_space(3))) void *)(tile + WHICH * geo::kTile + i * 1024), 16,
            lane_off[i], head_bytes, 0, kStreamOnce);
    if (FP8)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            scale_rsrc,
            (__attribute__((address_space(3))) void *)(tile + 2 * geo::kTile + WHICH * geo::kScaleSlot), 4,
            s_lane, scale_bytes, 0, 0);
    asm volatile("" ::: "memory");
}

// Wait until at most `groups` page-load groups (the newest ones) are still in
// flight.  Loads return in order, so everything issued before them has landed.
template <bool FP8>
__device__ __forceinline__ void wait_groups(int groups)
{
#define ADR_WAIT_CASE(N)                                                                          \
    case N:                                                                                       \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N * Geo<FP8>::kGroup) : "memory");                \
        break;
    switch (groups) {
        ADR_WAIT_CASE(6)
        ADR_WAIT_CASE(5)
        ADR_WAIT_CASE(4)
        ADR_WAIT_CASE(3)
        ADR_WAIT_CASE(2)
        ADR_WAIT_CASE(1)
    default:
        ADR_WAIT_CASE(0)
    }
#undef ADR_WAIT_CASE
}

// Two pages at once (page A, and page B = the wave's next page, 64 tokens further
// on): S = K Q^T for both, one online-softmax step over the 32 tokens, O += P V
// with the contraction running over both pages.  Only B can be the partition's
// last, partly filled page.  The work comes in four pieces so that the caller can
// issue loads between them.
struct PairWeights {
    u32x4 ah, al; // eight bf16 each: elements 0..3 <-> page A tokens 4j+i, 4..7 <-> page B tokens 4j+i
};

__device__ __forceinline__ void pair_scores(f32x4 &sa, f32x4 &sb, const u32x4 (&ka)[4],
                                            const u32x4 (&kb)[4], const u32x4 (&qb)[4])
{
    sa = f32x4{0.f, 0.f, 0.f, 0.f};
    sb = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kk]),
                                                     __builtin_bit_cast(bf16x8, qb[kk]), sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[kk]),
                                                     __builtin_bit_cast(bf16x8, qb[kk]), sb, 0, 0, 0);
    }
}

__device__ __forceinline__ PairWeights pair_softmax(WaveState &st, PageRegs &pb, f32x4 sa, f32x4 sb,
                                                    float score_a, float score_b, float p_scale_a,
                                                    float p_scale_b, int tok_b, int t1, int j)
{
    // tok_b = index of the first of this lane's four tokens in page B
    const bool tail = tok_b - 4 * j + kPageSize > t1;
    float sc[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sc[i] = sa[i] * score_a;
        sc[4 + i] = sb[i] * score_b;
        if (tail && tok_b + i >= t1)
            sc[4 + i] = -INFINITY;
    }
    if (tail) { // rows of tokens past the end may hold anything: keep them out of P*V
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (tok_b + u >= t1)
                pb.v[u] = u32x4{0u, 0u, 0u, 0u};
    }

    float bm = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])),
                     fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
    bm = max_across_rows(bm);
    if (__any(bm > st.m + kMaxSlack)) {
        const float mn = fmaxf(st.m, bm);
        const float alpha = fast_exp2(st.m - mn);
        st.m = mn;
        st.l *= alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = __shfl(alpha, 4 * j + i);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                st.o[e][i] *= a;
        }
    }
    uint32_t ph[8], pl[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float pw = fast_exp2(sc[i] - st.m);
        st.l += pw;
        pw *= i < 4 ? p_scale_a : p_scale_b;
        ph[i] = __float_as_uint(pw) & 0xffff0000u;            // bf16 head (truncated)
        pl[i] = __float_as_uint(pw - __uint_as_float(ph[i])); // remainder, exact in fp32
    }
    PairWeights w;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        w.ah[h] = (ph[2 * h] >> 16) | ph[2 * h + 1];
        w.al[h] = (pl[2 * h] >> 16) | (pl[2 * h + 1] & 0xffff0000u);
    }
    return w;
}

template <int E0, int E1>
__device__ __forceinline__ void pair_pv(WaveState &st, const PairWeights &w, const PageRegs &pa,
                                        const PageRegs &pb)
{
#pragma unroll
    for (int e = E0; e < E1; ++e) {
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        u32x4 vb;
        vb[0] = __builtin_amdgcn_perm(pa.v[1][e >> 1], pa.v[0][e >> 1], sel);
        vb[1] = __builtin_amdgcn_perm(pa.v[3][e >> 1], pa.v[2][e >> 1], sel);
        vb[2] = __builtin_amdgcn_perm(pb.v[1][e >> 1], pb.v[0][e >> 1], sel);
        vb[3] = __builtin_amdgcn_perm(pb.v[3][e >> 1], pb.v[2][e >> 1], sel);
        st.o[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, w.ah), __builtin_bit_cast(bf16x8, vb), st.o[e], 0, 0, 0);
        st.o[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, w.al), __builtin_bit_cast(bf16x8, vb), st.o[e], 0, 0, 0);
    }
}

// Read one ring stage into operand registers (widening an fp8 page to bf16).
template <bool FP8>
__device__ __forceinline__ void read_stage(const char *tile, const uint32_t (&k_read)[4], uint32_t v_read,
                                           PageRegs &pr, u32x4 (&ka)[4], float &k_scale, float &v_scale)
{
    typedef Geo<FP8> geo;
    if (FP8) {
        u32x2 vraw[4], kraw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            vraw[u] = *(const u32x2 *)(tile + geo::kTile + v_read + u * geo::kRow);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            kraw[kk] = *(const u32x2 *)(tile + k_read[kk]);
        k_scale = *(const float *)(tile + 2 * geo::kTile);
        v_scale = *(const float *)(tile + 2 * geo::kTile + geo::kScaleSlot);
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
        k_scale = v_scale = 1.f;
    }
}

// ---- fp8 cache: operands without widening K, V read transposed -----------------------------
// K: the bytes of an fp8 K tile feed v_mfma_f32_16x16x32_fp8_fp8 as they are (lane (r, j) holds 8
// bytes of token r), against the query split into two fp8 numbers per element (below), so that
// nothing of K is ever widened.
//
// V: the B operand of O += P V wants lane (n, j) to hold, for ONE column n, the values of eight
// tokens -- the transpose of how a V tile lies in memory and in LDS.  gfx950 reads LDS transposed:
// with ds_read_b64_tr_b8 each lane of a group of sixteen names 8 bytes, and lane i receives byte
// i % 8 of the pieces named by lanes i / 8 + 2k, k = 0 .. 7.  So when lane h + 2k names "token
// T(k), columns 16e + 8h .. 16e + 8h + 7", with T = tokens 4j .. 4j + 3 of the pair's first page
// for k < 4 and of its second page for k >= 4, lane n receives column 16e + n of those eight tokens:
// the operand for column block e, widened to bf16 without any shuffling in registers.  The
// accumulator st.o[e] then holds O[head 4j + i][16e + n] in lane (n, j) (a bf16 cache, whose V
// operand is put together from plain reads by byte permutes, has O[head 4j + i][8n + e] there).
// Both fp8 tiles are stored with slot c of row t holding chunk c ^ (t & 7), so that the rows these
// reads touch fall into different LDS banks.
typedef long i64_t;

struct QueryFp8 {
    u32x2 hi[4], lo[4]; // q * 2^s = hi + lo, both E4M3 (exact for all but the smallest elements of a row)
    float unscale;      // 2^-s, this lane's head
};

// The transposed reads are written by hand, all eight of a step in one statement, and nothing waits for
// them there: the compiler would guard each one (it cannot tell the read's target from the ring
// slots that direct-to-LDS loads are still filling) with a wait for EVERY load in flight, which
// is exactly what the ring must not do.  The stage read here has landed (wait_groups); the results
// are valid after the caller's wait for the LDS (settle_copies below), which takes them as operands
// so that nothing reads them earlier.
__device__ __forceinline__ void lds_read_tr8_x8(const uint32_t (&addr)[8], u32x2 (&v)[8])
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("ds_read_b64_tr_b8 %0, %8 offset:%16\n\t"
                 "ds_read_b64_tr_b8 %1, %9 offset:%16\n\t"
                 "ds_read_b64_tr_b8 %2, %10 offset:%16\n\t"
                 "ds_read_b64_tr_b8 %3, %11 offset:%16\n\t"
                 "ds_read_b64_tr_b8 %4, %12 offset:%16\n\t"
                 "ds_read_b64_tr_b8 %5, %13 offset:%16\n\t"
                 "ds_read_b64_tr_b8 %6, %14 offset:%16\n\t"
                 "ds_read_b64_tr_b8 %7, %15 offset:%16"
                 : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
                 : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3]), "v"(addr[4]), "v"(addr[5]), "v"(addr[6]),
                   "v"(addr[7]), "n"(Geo<true>::kTile)
                 : "memory");
#else
    for (int e = 0; e < 8; ++e)
        v[e] = u32x2{addr[e], 0u};
#endif
}

// Wait for every LDS read of this wave.  What was read (transposed V pieces, K bytes, scales) goes
// through the statement, so that no use of it is scheduled above the wait, and the compiler, which
// inserts its own waits for the reads it knows of in front of this statement, has none left to
// place later on, where a wait for an LDS read would also wait for a page-table entry that is
// still on its way.
__device__ __forceinline__ void settle_copies(u32x2 (&v8)[8], u32x2 (&ka)[4], float &s0, float &s1)
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(v8[0]), "+v"(v8[1]), "+v"(v8[2]), "+v"(v8[3]), "+v"(v8[4]), "+v"(v8[5]), "+v"(v8[6]),
                   "+v"(v8[7]), "+v"(ka[0]), "+v"(ka[1]), "+v"(ka[2]), "+v"(ka[3]), "+v"(s0), "+v"(s1)
                 :
                 : "memory");
}

__device__ __forceinline__ void settle_copies(u32x2 (&v8)[8], u32x2 (&ka)[4], u32x2 (&kb)[4], float &s0, float &s1,
                                              float &s2, float &s3)
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(v8[0]), "+v"(v8[1]), "+v"(v8[2]), "+v"(v8[3]), "+v"(v8[4]), "+v"(v8[5]), "+v"(v8[6]),
                   "+v"(v8[7]), "+v"(ka[0]), "+v"(ka[1]), "+v"(ka[2]), "+v"(ka[3]), "+v"(kb[0]), "+v"(kb[1]),
                   "+v"(kb[2]), "+v"(kb[3]), "+v"(s0), "+v"(s1), "+v"(s2), "+v"(s3)
                 :
                 : "memory");
}

__device__ __forceinline__ f32x4 mfma_fp8(u32x2 a, u32x2 b, f32x4 c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(__builtin_bit_cast(i64_t, a), __builtin_bit_cast(i64_t, b), c, 0, 0, 0);
#else
    return c;
#endif
}

// The query rows of an item as fp8 operands: every element is scaled by a power of two chosen per
// head (the head's largest element lands in [128, 256)) and split into an E4M3 number and the E4M3
// remainder; bf16 has eight significant bits, the two parts four each, so the split is exact except
// for elements 2^9 times smaller than the row's largest, which lose low bits worth 2^-17 of that
// largest element.  The scores are multiplied by 2^-s afterwards.
__device__ __forceinline__ QueryFp8 query_fp8(const u32x4 (&raw)[4])
{
    QueryFp8 q;
#if defined(__HIP_DEVICE_COMPILE__)
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    float amax = 0.f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int w = 0; w < 4; ++w)
            amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(raw[kk][w])), fabsf(bf16_hi(raw[kk][w]))));
    amax = max_across_rows(amax); // the head's 128 elements sit in the four lanes (r, 0 .. 3)
    const uint32_t e = (__float_as_uint(amax) >> 23) & 255u; // biased exponent of the largest element
    const bool plain = e < 8u || e > 246u;                   // zero, tiny or non-finite rows: no scaling
    const float scale = plain ? 1.f : __uint_as_float((261u - e) << 23); // 2^(134 - e)
    q.unscale = plain ? 1.f : __uint_as_float((e - 7u) << 23);          // 2^(e - 134)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        int hi[2] = {0, 0}, lo[2] = {0, 0};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float x0 = bf16_lo(raw[kk][w]) * scale, x1 = bf16_hi(raw[kk][w]) * scale;
            const bool upper = (w & 1) != 0;
            hi[w >> 1] = upper ? __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, hi[w >> 1], true)
                               : __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, hi[w >> 1], false);
            const f32x2 back = upper ? __builtin_amdgcn_cvt_pk_f32_fp8(hi[w >> 1], true)
                                     : __builtin_amdgcn_cvt_pk_f32_fp8(hi[w >> 1], false);
            lo[w >> 1] = upper ? __builtin_amdgcn_cvt_pk_fp8_f32(x0 - back[0], x1 - back[1], lo[w >> 1], true)
                               : __builtin_amdgcn_cvt_pk_fp8_f32(x0 - back[0], x1 - back[1], lo[w >> 1], false);
        }
        q.hi[kk] = u32x2{(uint32_t)hi[0], (uint32_t)hi[1]};
        q.lo[kk] = u32x2{(uint32_t)lo[0], (uint32_t)lo[1]};
    }
#else
    (void)raw;
    q.unscale = 1.f;
#endif
    return q;
}

// K bytes and the two scales of one fp8 ring stage.
__device__ __forceinline__ void read_stage_fp8(const char *tile, const uint32_t (&k_read)[4], u32x2 (&k8)[4],
                                               float &k_scale, float &v_scale)
{
    typedef Geo<true> geo;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        k8[kk] = *(const u32x2 *)(tile + k_read[kk]);
    k_scale = *(const float *)(tile + 2 * geo::kTile);
    v_scale = *(const float *)(tile + 2 * geo::kTile + geo::kScaleSlot);
}

// The V bytes of a pair of pages (or of one page, when both stages are the same), given the stages'
// byte offsets in the wave's ring: lanes whose piece belongs to the second page (`second`) name that
// stage.
__device__ __forceinline__ void read_v8(const char *ring, int stage_a, int stage_b, bool second,
                                        const uint32_t (&vt_off)[8], u32x2 (&v8)[8])
{
    const uint32_t base = lds_address(ring) + (uint32_t)(second ? stage_b : stage_a);
    uint32_t addr[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
        addr[e] = base + vt_off[e];
    lds_read_tr8_x8(addr, v8);
}

__device__ __forceinline__ void pair_scores_fp8(f32x4 &sa, f32x4 &sb, const u32x2 (&ka)[4], const u32x2 (&kb)[4],
                                                const QueryFp8 &q)
{
    sa = f32x4{0.f, 0.f, 0.f, 0.f};
    sb = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        sa = mfma_fp8(ka[kk], q.hi[kk], sa);
        sb = mfma_fp8(kb[kk], q.hi[kk], sb);
        sa = mfma_fp8(ka[kk], q.lo[kk], sa);
        sb = mfma_fp8(kb[kk], q.lo[kk], sb);
    }
}

// A word of four bytes that clears, in a V operand, the tokens of this lane at or past t1 (tok =
// index of the lane's first token).
__device__ __forceinline__ uint32_t tail_mask_fp8(int tok, int t1)
{
    return (tok + 0 < t1 ? 0x000000ffu : 0u) | (tok + 1 < t1 ? 0x0000ff00u : 0u) | (tok + 2 < t1 ? 0x00ff0000u : 0u) |
           (tok + 3 < t1 ? 0xff000000u : 0u);
}

// O += P V over two pages, column blocks E0 .. E1 - 1; v8: the pair's bytes (four tokens of the
// first page, then four of the second, per column), widened here.
template <int E0, int E1>
__device__ __forceinline__ void pair_pv_fp8(WaveState &st, const PairWeights &w, const u32x2 (&v8)[8])
{
#pragma unroll
    for (int e = E0; e < E1; ++e) {
        const u32x4 b = fp8x8_to_bf16x8(v8[e]);
        st.o[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w.ah), __builtin_bit_cast(bf16x8, b),
                                                          st.o[e], 0, 0, 0);
        st.o[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w.al), __builtin_bit_cast(bf16x8, b),
                                                          st.o[e], 0, 0, 0);
    }
}

// One fp8 page on its own: the same steps over 16 tokens, P V as 16x16x16 products.  v8: a transposed
// read whose first four tokens are the page's.
__device__ __forceinline__ void single_page_fp8(WaveState &st, const u32x2 (&k8)[4], const u32x2 (&v8)[8],
                                                const QueryFp8 &q, float score_scale, float p_scale, int tok, int t1,
                                                int j)
{
    f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        s = mfma_fp8(k8[kk], q.hi[kk], s);
        s = mfma_fp8(k8[kk], q.lo[kk], s);
    }
    const bool tail = tok - 4 * j + kPageSize > t1;
    float sc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sc[i] = s[i] * score_scale;
        if (tail && tok + i >= t1)
            sc[i] = -INFINITY;
    }
    float bm = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
    bm = max_across_rows(bm);
    if (__any(bm > st.m + kMaxSlack)) {
        const float mn = fmaxf(st.m, bm);
        const float alpha = fast_exp2(st.m - mn);
        st.m = mn;
        st.l *= alpha;
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
        ph[i] = __float_as_uint(pw) & 0xffff0000u;
        pl[i] = __float_as_uint(pw - __uint_as_float(ph[i]));
    }
    u32x2 ah, al;
    ah[0] = (ph[0] >> 16) | ph[1];
    ah[1] = (ph[2] >> 16) | ph[3];
    al[0] = (pl[0] >> 16) | (pl[1] & 0xffff0000u);
    al[1] = (pl[2] >> 16) | (pl[3] & 0xffff0000u);
    const uint32_t keep = tail ? tail_mask_fp8(tok, t1) : 0xffffffffu; // rows past the end may hold anything
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const u32x4 wide = fp8x8_to_bf16x8(u32x2{v8[e][0] & keep, 0u});
        const u32x2 b = u32x2{wide[0], wide[1]};
        st.o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, ah), __builtin_bit_cast(s16x4, b),
                                                            st.o[e], 0, 0, 0);
        st.o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, al), __builtin_bit_cast(s16x4, b),
                                                            st.o[e], 0, 0, 0);
    }
}

// STAGES > 0 fixes the ring depth at compile time (the depths of the common shapes: ring
// positions and wait counts become constants); STAGES = 0 takes it from the parameters.
// An fp8 pass runs two workgroups per compute unit, i.e. two waves per SIMD: its register
// budget is half the file.
template <bool FP8, int STAGES>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(FP8 ? 2 : 1, 2)))
void decode_stream_kernel(const StreamParams sp)
{
    typedef Geo<FP8> geo;
    constexpr int kStageBytes = geo::kStage;
    const DecodeParams &p = sp.d;
    const int S = STAGES > 0 ? STAGES : sp.stages;
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const int ring_bytes = kWaves * S * kStageBytes;
    const int qtile_bytes = sp.q_rows * (D * 2);
    Shared &sh = *(Shared *)(lds_raw + ring_bytes + kWaves * qtile_bytes);
    float *staging = (float *)((char *)&sh + sizeof(Shared)); // [nb][kWaves][G][D]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15;
    const int j = lane >> 4;
    const int B = p.B, Hkv = p.Hkv, G = p.G;

    // The first three tickets: drawn before anything else, so that the round trip
    // overlaps the scan below.
    uint32_t first_ticket = 0;
    if (tid == 0)
        asm volatile("s_nop 4\n\tglobal_atomic_add %0, %1, %2, %3 sc0"
                     : "=&v"(first_ticket)
                     : "v"(0), "v"(3), "s"(sp.ctl)
                     : "memory");

    // ---- partitions per row: exclusive prefix sums over the rows, four rows per thread
    int cshift = 0, total_full = 0, total_rag = 0;
    {
        int len4[4]; // this thread's rows; read without a condition (a row past the end re-reads the
                     // last one), so that the four reads are in flight together
#pragma unroll
        for (int i = 0; i < 4; ++i)
            len4[i] = p.seq_lens[min(tid * 4 + i, B - 1)];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = tid * 4 + i;
            len4[i] = row < B ? max(min(len4[i], p.max_seq_len), 0) : -1;
        }
        if (tid < kQueue)
            sh.rec[tid].seq = -1;
        if (tid == 0) {
            sh.gen[0] = sh.gen[1] = 0;
            sh.arrive[0] = sh.arrive[1] = 0;
            sh.failed = 0;
        }
        // items of `pt` tokens: full ones per row, and one ragged (or empty) last one where there is one
        auto scan_rows = [&](int pt) {
            int f[4], g[4], sf = 0, sg = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int L = len4[i];
                f[i] = L >= 0 ? L / pt : 0;
                g[i] = L >= 0 && (L % pt != 0 || L == 0) ? 1 : 0; // an empty row still owns one (empty) item
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
            }
            __syncthreads();
        };
        scan_rows(sp.pt);
        // Many items: hand out runs of two or four partitions as one item.  What an item costs
        // besides its pages (records, staging, combining) is then paid half or a quarter as
        // often, and there are still enough items to balance the workgroups.  The run's result
        // goes to its first partition's place and the others are marked empty, which the merge
        // skips.  The threshold counts items, not workgroups, so the choice (and with it the
        // order of the floating-point sums) depends on the inputs alone.
        if (p.coalesce && p.partition_tokens > 0 && sp.pt <= (1 << 24)) {
            const int64_t items = ((int64_t)sh.total[0] + sh.total[1]) * Hkv;
            cshift = items >= 4 * kCoalesceItems ? 2 : items >= 2 * kCoalesceItems ? 1 : 0;
            cshift = __builtin_amdgcn_readfirstlane(cshift);
            if (cshift)
                scan_rows(sp.pt << cshift);
        }
        total_full = __builtin_amdgcn_readfirstlane(sh.total[0]);
        total_rag = __builtin_amdgcn_readfirstlane(sh.total[1]);
        if (tid == 0) {
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(first_ticket)::"memory");
            sh.first[0] = (int)first_ticket;
            sh.first[1] = (int)first_ticket + 1;
            sh.first[2] = (int)first_ticket + 2;
        }
        __syncthreads();
        if (wave < 3)
            publish(sh.rec[wave], decode_ticket(sh, sp, sh.first[wave], cshift, total_full, total_rag), wave);
        __syncthreads();
    }

    // ---- per-lane constants
    // bf16: a row is sixteen 16-byte chunks and a load covers four rows; slot c of row t
    //       holds chunk c ^ t.  Step kk of QK^T reads chunk kk*4 + j of row r (8 elements).
    // fp8:  a row is eight 16-byte chunks and a load covers eight rows; slot c of row t
    //       holds chunk c ^ (t & 7), in the K tile and in the V tile.  The same 8 elements are the
    //       8-byte piece kk*4 + j.
    const uint32_t tok_bytes = (uint32_t)Hkv * geo::kRow;
    const uint32_t page_bytes = kPageSize * tok_bytes;
    const int rq = r < G ? r : 0; // query row this lane reads (columns >= G repeat head 0 and are never stored)
    uint32_t k_lane[4], v_lane[4], q_lane[4], k_read[4], q_read[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = 4 * i + j; // query-tile row this lane fetches in load i
        q_lane[i] = t * (D * 2) + ((r ^ t) * 16);
        q_read[i] = rq * (D * 2) + (((i * 4 + j) ^ rq) * 16);
        if (FP8) {
            const int tf = 8 * (i & 1) + (lane >> 3), c = lane & 7; // row / slot of load i (i < 2)
            k_lane[i] = tf * tok_bytes + ((c ^ (tf & 7)) * 16);
            v_lane[i] = k_lane[i];
            const int piece = i * 4 + j;
            k_read[i] = r * D + (((piece >> 1) ^ (r & 7)) * 16) + (piece & 1) * 8;
        } else {
            k_lane[i] = t * tok_bytes + ((r ^ t) * 16);
            v_lane[i] = t * tok_bytes + r * 16;
            k_read[i] = r * (D * 2) + (((i * 4 + j) ^ r) * 16);
        }
    }
    // V operand, bf16: rows 4j + u, the 8 elements 8r .. 8r+7
    const uint32_t v_read = (4 * j) * geo::kRow + r * (geo::kRow / 16);
    // V operand, fp8, read transposed: lane h + 2k of its group of sixteen names the 8 bytes "token
    // 4j + (k & 3) of the pair's first (k < 4) or second page, columns 16e + 8h .. +7": half h of
    // chunk e, which sits in slot e ^ (t & 7) of the token's row.
    uint32_t vt_off[8];
    const bool vt_second = (r >> 1) >= 4;
    {
        const int vt_row = 4 * j + ((r >> 1) & 3);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            vt_off[e] = vt_row * geo::kRow + ((e ^ (vt_row & 7)) << 4) + 8 * (r & 1);
    }
    const uint32_t s_lane = lane == 0 ? 0u : 0x7ffffff0u; // scale loads: only lane 0 is in range
    const char *kc = (const char *)p.k_cache;
    const char *vc = (const char *)p.v_cache;
    char *ring = lds_raw + wave * (S * kStageBytes);
    char *myq = lds_raw + ring_bytes + wave * qtile_bytes;
    const __amdgpu_buffer_rsrc_t null_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)kc, 0, 0, 0x00020000); // every read is out of range: zeros
    const int scale_range = FP8 ? p.num_pages * Hkv * 4 : 0;
    const __amdgpu_buffer_rsrc_t ks_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(FP8 ? (const void *)p.k_scale : (const void *)kc), 0, scale_range, 0x00020000);
    const __amdgpu_buffer_rsrc_t vs_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(FP8 ? (const void *)p.v_scale : (const void *)kc), 0, scale_range, 0x00020000);
    const int pages_per_part = (sp.pt << cshift) / kPageSize; // 2^26 when the pass is not split (part is 0 then)
    // "Page" below is a 16-token tile of the pool; a cache page is 1 << tsh of them (the
    // instantiations with a fixed ring depth serve 16-token pages only).
    const int tsh = STAGES > 0 ? 0 : p.page_shift;

    const Waits waits = {&sh.failed, p.spin_limit};
    Item C = fetch(sh.rec[0], 0, waits);
    Item N = fetch(sh.rec[1], 1, waits);
    issue_query(myq, sp, C, q_lane);

    // ---- load cursor: the next page of this wave's stream to be issued.  It runs
    // through the current item and on into the next one, never further.  It keeps
    // its own copy of what it needs from the item it is in.
#define ADR_FIRST_PAGE(IT) ((IT).part * pages_per_part + wave)
#define ADR_END_PAGE(IT) ((IT).valid ? ((IT).t1 + kPageSize - 1) / kPageSize : 0)
    int ld_in_next = 0;
    int ld_pg = ADR_FIRST_PAGE(C), ld_end = ADR_END_PAGE(C);
    uint32_t ld_head = (uint32_t)C.kvh * geo::kRow;
    int ld_kvh = C.kvh;
    table_ptr ld_bt = (table_ptr)(p.block_table + (int64_t)C.b * p.max_pages);
    int ld_ok = 0, ld_entry = 0; // ld_entry: the table's entry for the cursor's page, as loaded
#ifdef ADR_DEBUG_BOUNDS /* the row the cursor is in, for the record of an out-of-pool page id */
#define ADR_CURSOR_ROW (int)((ld_bt - (table_ptr)p.block_table) / p.max_pages)
#else
#define ADR_CURSOR_ROW 0
#endif
#define ADR_SETTLE()                                                                              \
    do { /* move the cursor to the next existing page and fetch its table entry (not looked at    \
            before the page is issued: the load is given the time until then) */                  \
        if (!ld_in_next && ld_pg >= ld_end) {                                                     \
            ld_in_next = 1;                                                                       \
            ld_pg = ADR_FIRST_PAGE(N);                                                            \
            ld_end = ADR_END_PAGE(N);                                                             \
            ld_head = (uint32_t)N.kvh * geo::kRow;                                                \
            ld_kvh = N.kvh;                                                                       \
            ld_bt = (table_ptr)(p.block_table + (int64_t)N.b * p.max_pages);                      \
        }                                                                                         \
        ld_ok = (unsigned)ld_pg < (unsigned)ld_end;                                               \
        if (ld_ok)                                                                                \
            ld_entry = ld_bt[ld_pg >> tsh];                                                       \
    } while (0)
    // Ring state: `occ` slots starting at `head` are occupied, in issue order; the
    // next load group goes to `tail`.  real_mask marks the slots that hold a page.
    int head = 0, tail = 0, occ = 0, real_mask = 0;
    int age = 0; // page-load groups issued since this item's look-ahead loads
    // A page is issued in two halves (K, then V); the second half takes the page
    // from the pend_* copies, because the cursor has moved on by then.
    char *pend_tile = ring;
    int pend_ok = 0, pend_id = 0;
    uint32_t pend_head = 0, pend_scale = 0;
#define ADR_ISSUE_K()                                                                             \
    do { /* the ring's tail slot takes the cursor's page, or a group of null loads: K half */     \
        pend_tile = ring + tail * kStageBytes;                                                    \
        pend_ok = ld_ok;                                                                          \
        if (ld_ok) {                                                                              \
            pend_id = pool_tile_checked(ld_entry, ld_pg, p.num_pages, tsh, p.bounds,              \
                                        ADR_CURSOR_ROW);                                          \
            pend_head = ld_head;                                                                  \
            pend_scale = (uint32_t)((pend_id >> tsh) * Hkv + ld_kvh) * 4u;                        \
            issue_half<FP8, 0>(pend_tile, page_rsrc(kc, pend_id, page_bytes), ks_rsrc, k_lane,    \
                               s_lane, pend_head, pend_scale);                                    \
            real_mask |= 1 << tail;                                                               \
            ld_pg += kWaves;                                                                      \
            ADR_SETTLE();                                                                         \
        } else {                                                                                  \
            issue_half<FP8, 0>(pend_tile, null_rsrc, null_rsrc, k_lane, s_lane, 0, 0);            \
            real_mask &= ~(1 << tail);                                                            \
        }                                                                                         \
        tail = tail + 1 == S ? 0 : tail + 1;                                                      \
        ++occ;                                                                                    \
        ++age;                                                                                    \
    } while (0)
#define ADR_ISSUE_V()                                                                             \
    do { /* V half of the page whose K half was issued last */                                    \
        if (pend_ok)                                                                              \
            issue_half<FP8, 1>(pend_tile, page_rsrc(vc, pend_id, page_bytes), vs_rsrc, v_lane,    \
                               s_lane, pend_head, pend_scale);                                    \
        else                                                                                      \
            issue_half<FP8, 1>(pend_tile, null_rsrc, null_rsrc, v_lane, s_lane, 0, 0);            \
    } while (0)
#define ADR_ISSUE()                                                                               \
    do {                                                                                          \
        ADR_ISSUE_K();                                                                            \
        ADR_ISSUE_V();                                                                            \
    } while (0)
    ADR_SETTLE();
    // Fill the ring behind the first item's query rows; once no more than the ring's
    // loads are in flight, those rows have landed.
    while (occ < S)
        ADR_ISSUE();
    wait_groups<FP8>(S);

    uint32_t next_ticket = 0;
    int invalid_run = 0;
    Item P = C; // the item before the current one (combined one item late); not read before it is one
    P.valid = 0;
    // Tickets are drawn by four different waves at their own pace, so a ticket past
    // the end can precede a valid one in the queue; each wave's own draws are in
    // order, so four invalid records in a row mean the work is finished.
    for (int k = 0;; ++k) {
        invalid_run = C.valid ? 0 : invalid_run + 1;
        if (invalid_run == kWaves)
            break;
        // ---- this item's query rows leave the wave's tile for registers (they landed before the
        // previous item ended); the tile is then free for the next item's rows.
        u32x4 qb[4]; // B operand of QK^T: head r's query, chunk order matching the K reads
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            qb[kk] = *(const u32x4 *)(myq + q_read[kk]);
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(qb[0]), "+v"(qb[1]), "+v"(qb[2]), "+v"(qb[3])::"memory");
        // ---- look-ahead loads: the query rows of the next item, and (one wave) the
        // ticket of the item three ahead.  The counter's address may reach its scalar
        // registers through a vector-lane read just before the statement; the five
        // wait states such a value needs before a memory instruction may use it are
        // not inserted around hand-written instructions, hence the s_nop.
        const bool drawer = (k & (kWaves - 1)) == wave;
        issue_query(myq, sp, N, q_lane);
        if (drawer && lane == 0)
            asm volatile("s_nop 4\n\tglobal_atomic_add %0, %1, %2, %3 sc0"
                         : "=&v"(next_ticket)
                         : "v"(0), "v"(1), "s"(sp.ctl)
                         : "memory");
        age = 0;

        WaveState st;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            st.o[e] = f32x4{0.f, 0.f, 0.f, 0.f};
        st.m = kNegBig;
        st.l = 0.f;
        QueryFp8 q8; // fp8 cache: the same query as two fp8 numbers per element
        float q_score = p.scale_log2e;
        if constexpr (FP8) {
            q8 = query_fp8(qb);
            q_score *= q8.unscale;
        }

        const int pg_end = ADR_END_PAGE(C);
        for (int pg = ADR_FIRST_PAGE(C); pg < pg_end;) {
            // Fill the ring, then pass over null slots at its head: each one frees a
            // slot for the page the cursor now has.  The page wanted here is in the
            // ring or at the cursor, so this ends after at most S steps.
            while (occ < S)
                ADR_ISSUE();
            for (int guard = 0; !((real_mask >> head) & 1) && guard <= S; ++guard) {
                head = head + 1 == S ? 0 : head + 1;
                --occ;
                ADR_ISSUE();
            }
            if (!((real_mask >> head) & 1)) { // cannot happen; never consume a slot that holds no page
                count_fault(waits);
                pg += kWaves;
                continue;
            }
            const int second = head + 1 == S ? 0 : head + 1;
            const bool pair = pg + kWaves < pg_end && ((real_mask >> second) & 1);
            // the ring is full: S - 1 groups are newer than the head's, S - 2 newer than its successor's
            wait_groups<FP8>(pair ? S - 2 : S - 1);
            if constexpr (FP8) {
                // Copy the stage(s) to registers (the K bytes as they are, the V bytes transposed), hand the
                // slots straight back to the ring and refill them, so that the loads are under way while
                // this step computes.
                u32x2 ka8[4], v8[8];
                float ks_a, vs_a;
                const int stage_a = head * kStageBytes;
                read_stage_fp8(ring + stage_a, k_read, ka8, ks_a, vs_a);
                if (pair) {
                    u32x2 kb8[4];
                    float ks_b, vs_b;
                    const int stage_b = second * kStageBytes;
                    read_stage_fp8(ring + stage_b, k_read, kb8, ks_b, vs_b);
                    read_v8(ring, stage_a, stage_b, vt_second, vt_off, v8);
                    settle_copies(v8, ka8, kb8, ks_a, vs_a, ks_b, vs_b); // the copies are complete
                    f32x4 sa, sb;
                    const int tok_b = (pg + kWaves) * kPageSize + 4 * j;
                    PageRegs none; // (the V bytes are masked below, not inside the softmax step)
                    real_mask &= ~((1 << head) | (1 << second));
                    head = second + 1 == S ? 0 : second + 1;
                    occ -= 2;
                    ADR_ISSUE_K();
                    pair_scores_fp8(sa, sb, ka8, kb8, q8);
                    ADR_ISSUE_V();
                    const PairWeights w =
                        pair_softmax(st, none, sa, sb, q_score * ks_a, q_score * ks_b, vs_a, vs_b, tok_b, C.t1, j);
                    if (tok_b - 4 * j + kPageSize > C.t1) { // rows of tokens past the end may hold anything
                        const uint32_t keep = tail_mask_fp8(tok_b, C.t1);
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            v8[e][1] &= keep;
                    }
                    ADR_ISSUE_K();
                    pair_pv_fp8<0, 4>(st, w, v8);
                    ADR_ISSUE_V();
                    pair_pv_fp8<4, 8>(st, w, v8);
                    pg += 2 * kWaves;
                } else {
                    read_v8(ring, stage_a, stage_a, false, vt_off, v8); // its first four tokens are the page's
                    settle_copies(v8, ka8, ks_a, vs_a);
                    real_mask &= ~(1 << head);
                    head = second;
                    occ -= 1;
                    while (occ < S)
                        ADR_ISSUE();
                    single_page_fp8(st, ka8, v8, q8, q_score * ks_a, vs_a, pg * kPageSize + 4 * j, C.t1, j);
                    pg += kWaves;
                }
            } else {
            // Copy the stage(s) to registers, hand the slots straight back to the ring and
                // refill them, so that the loads are under way while this step computes.
                PageRegs pa;
                u32x4 ka[4];
                float ks_a, vs_a;
                read_stage<FP8>(ring + head * kStageBytes, k_read, v_read, pa, ka, ks_a, vs_a);
                if (pair) {
                    PageRegs pb;
                    u32x4 kb[4];
                    float ks_b, vs_b;
                    read_stage<FP8>(ring + second * kStageBytes, k_read, v_read, pb, kb, ks_b, vs_b);
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the copies are complete
                    // the two freed slots are refilled in four pieces between the pieces of the arithmetic
                    f32x4 sa, sb;
                    real_mask &= ~((1 << head) | (1 << second));
                    head = second + 1 == S ? 0 : second + 1;
                    occ -= 2;
                    ADR_ISSUE_K();
                    pair_scores(sa, sb, ka, kb, qb);
                    ADR_ISSUE_V();
                    const PairWeights w = pair_softmax(st, pb, sa, sb, p.scale_log2e * ks_a, p.scale_log2e * ks_b,
                                                       vs_a, vs_b, (pg + kWaves) * kPageSize + 4 * j, C.t1, j);
                    ADR_ISSUE_K();
                    pair_pv<0, 4>(st, w, pa, pb);
                    ADR_ISSUE_V();
                    pair_pv<4, 8>(st, w, pa, pb);
                    pg += 2 * kWaves;
                } else {
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    real_mask &= ~(1 << head);
                    head = second;
                    occ -= 1;
                    while (occ < S)
                        ADR_ISSUE();
                    attend_page(st, pa, ka, qb, p.scale_log2e * ks_a, vs_a, pg * kPageSize + 4 * j, C.t1, j);
                    pg += kWaves;
                }
            }
        }

        // ---- the look-ahead loads must have landed: they are older than the `age`
        // newest groups, and no more than S groups are ever in flight
        wait_groups<FP8>(min(age, S));
        asm volatile("" : "+v"(next_ticket)::"memory"); // the ticket is read after the wait, not before
        if (drawer)
            publish(sh.rec[(k + 3) & (kQueue - 1)],
                    decode_ticket(sh, sp, (int)__builtin_amdgcn_readfirstlane(next_ticket), cshift, total_full,
                                  total_rag),
                    k + 3);

        // ---- the record of the item after next and the state of this item's staging buffer, in one
        // LDS round trip (and ahead of the delivery, so that the item's last matrix instructions
        // drain behind it)
        const int buf = sp.nb == 2 ? (k & 1) : 0;
        const int use = sp.nb == 2 ? (k >> 1) : k;
        int gen_seen = 0;
        const Item after_next =
            fetch(sh.rec[(k + 2) & (kQueue - 1)], k + 2, waits, &sh.gen[buf], &gen_seen);
        if (gen_seen != use)
            poll_equal(&sh.gen[buf], use, waits); // the buffer's previous item has been combined

        // ---- deliver this wave's share (an item past the end still takes its turn of the buffers)
        if (C.valid) {
            float l = st.l;
            l = sum_across_rows(l);
            float *so = staging + (buf * kWaves + wave) * (G * D); // [G][D]
            if (j == 0 && r < G) {
                sh.ml[buf][wave][r][0] = st.m;
                sh.ml[buf][wave][r][1] = l;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int g = 4 * j + i;
                if (g < G) {
                    *(f32x4 *)(so + g * D + 8 * r) = f32x4{st.o[0][i], st.o[1][i], st.o[2][i], st.o[3][i]};
                    *(f32x4 *)(so + g * D + 8 * r + 4) = f32x4{st.o[4][i], st.o[5][i], st.o[6][i], st.o[7][i]};
                }
            }
        }
        lds_order();
        if (lane == 0)
            flag_add_async(&sh.arrive[buf], 1); // behind the writes above, in the LDS's order
        lds_order();

        // ---- combine.  The waves take turns (leaving it to the last one to arrive would load every
        // item's extra work on the wave the others are already waiting for).  With two staging
        // buffers the turn is one item late: at the end of item k the wave combines item k - 1,
        // which the other three have almost always delivered by then, so that nobody has to fall
        // in step with the slowest wave; with one buffer it combines item k and waits for them.
        const int late = sp.nb == 2 ? 1 : 0;
        if (((k + 2) & (kWaves - 1)) == wave && k >= late) {
            const Item &Q = late ? P : C;
            const int qbuf = late ? ((k - 1) & 1) : 0;
            const int quse = late ? ((k - 1) >> 1) : k;
            // Once a wait of this workgroup has expired (this one or an earlier one, of any wave), what
            // the staging buffers hold cannot be trusted: the item gets NaN instead.
            int failed_seen = 0;
            const bool arrived = poll_equal_also(&sh.arrive[qbuf], kWaves, waits, &sh.failed, &failed_seen);
            const bool bad = !arrived || failed_seen != 0;
            {
                if (Q.valid) {
                    // Two output quads per lane and round; all LDS reads of a round are issued
                    // before anything is computed, so the round costs one LDS latency, not ten.
                    const float *sbase = staging + qbuf * kWaves * (G * D);
                    const int quads = G * (D / 4);
                    typedef float f32x2 __attribute__((ext_vector_type(2)));
                    for (int base = 0; base < quads; base += 128) {
                        bool ok[2];
                        int g[2], c4[2];
                        f32x2 ml[2][kWaves];
                        f32x4 x[2][kWaves];
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            const int idx = base + 64 * t + lane;
                            ok[t] = idx < quads;
                            g[t] = ok[t] ? idx / (D / 4) : 0;
                            c4[t] = (idx & (D / 4 - 1)) * 4;
#pragma unroll
                            for (int w = 0; w < kWaves; ++w) {
                                ml[t][w] = *(const f32x2 *)&sh.ml[qbuf][w][g[t]][0];
                                x[t][w] = *(const f32x4 *)(sbase + w * (G * D) + g[t] * D + c4[t]);
                            }
                        }
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            if (!ok[t])
                                continue;
                            float M = kNegBig;
#pragma unroll
                            for (int w = 0; w < kWaves; ++w)
                                M = fmaxf(M, ml[t][w][0]);
                            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
                            float den = 0.f;
#pragma unroll
                            for (int w = 0; w < kWaves; ++w) {
                                const float f = fast_exp2(ml[t][w][0] - M);
                                acc += f * x[t][w];
                                den += f * ml[t][w][1];
                            }
                            const float inv = den > 0.f ? 1.f / den : 0.f;
                            const float lse_ok = den > 0.f ? (M + fast_log2(den)) * kLn2 : -INFINITY;
                            const float lse = bad ? __builtin_nanf("") : lse_ok;
                            f32x4 o = acc * inv;
                            if (bad)
                                o = f32x4{lse, lse, lse, lse};
                            const int h = Q.kvh * G + g[t];
                            // fp8: the staged quad at place c4 = 8n + 4q holds columns 16 (4q + u) + n, u = 0 .. 3
                            // (four stores, each of which the sixteen lanes n fill 64 bytes of); bf16: columns
                            // c4 .. c4 + 3.
                            const int col = ((c4[t] & 4) << 4) + (c4[t] >> 3);
                            if (Q.n_parts == 1) {
                                const int64_t row_off = ((int64_t)Q.b * p.Hq + h) * D;
                                if constexpr (FP8) {
#pragma unroll
                                    for (int u = 0; u < 4; ++u) {
                                        if (p.out_f32)
                                            ((float *)p.out)[row_off + col + 16 * u] = o[u];
                                        else
                                            ((uint16_t *)p.out)[row_off + col + 16 * u] = (uint16_t)f32_to_bf16(o[u]);
                                    }
                                } else if (p.out_f32) {
                                    *(f32x4 *)((float *)p.out + row_off + c4[t]) = o;
                                } else {
                                    u32x2 packed;
                                    packed[0] = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
                                    packed[1] = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
                                    *(u32x2 *)((uint16_t *)p.out + row_off + c4[t]) = packed;
                                }
                                if (p.lse && c4[t] == 0)
                                    p.lse[(int64_t)Q.b * p.Hq + h] = lse;
                            } else {
                                const int64_t row = ((int64_t)Q.b * p.max_parts + (Q.part << cshift)) * p.Hq + h;
                                if constexpr (FP8) {
#pragma unroll
                                    for (int u = 0; u < 4; ++u)
                                        p.part_o[row * D + col + 16 * u] = o[u];
                                } else {
                                    *(f32x4 *)(p.part_o + row * D + c4[t]) = o;
                                }
                                if (c4[t] == 0)
                                    p.part_lse[row] = lse;
                            }
                        }
                    }
                    if (cshift && Q.n_parts > 1) {
                        // the other partitions of the run carry no mass: lse = -inf, payload never read
                        const int slot = (Q.part << cshift) + 1;
                        const int n = (min((Q.part + 1) << cshift, Q.n_parts) - slot) * G;
                        if (lane < n)
                            p.part_lse[((int64_t)Q.b * p.max_parts + slot + lane / G) * p.Hq + Q.kvh * G + lane % G] =
                                -INFINITY;
                    }
                }
                if (arrived && lane == 0) { // hand the buffer back
                    flag_write(&sh.arrive[qbuf], 0);
                    flag_write(&sh.gen[qbuf], quse + 1);
                }
            }
        }
        P = C;

        // ---- next item becomes current
        C = N;
        N = after_next;
        // The cursor is always inside the item that has just become current (issuing
        // the last page of an item moves it on, and so does an item without pages).
        ld_in_next = 0;
        if (!ld_ok)
            ADR_SETTLE(); // it had run out of pages there: move on into the new next item
    }

#undef ADR_ISSUE
#undef ADR_ISSUE_V
#undef ADR_ISSUE_K
#undef ADR_SETTLE
#undef ADR_CURSOR_ROW
#undef ADR_FIRST_PAGE
#undef ADR_END_PAGE

    // ---- hand the launch's control block back cleared once every workgroup is through.  (Every wave's
    // own fault counts have completed by now: they were waited for above the barrier.)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        int poison = 0;
        const uint32_t done = atomicAdd(sp.ctl + kLaunchFinished, 1u);
        if (done == gridDim.x - 1) {
            poison = atomicExch(sp.ctl + kLaunchExpired, 0u) != 0u;
            atomicExch(sp.ctl + kLaunchTicket, 0u);
            atomicExch(sp.ctl + kLaunchFinished, 0u);
        }
        sh.first[0] = poison;
    }
    __syncthreads();
    // A wait expired somewhere in this launch: no row of it may pass as a result.  (What this needs
    // of the parameters is read afresh from the kernel's argument block, so that none of it has to
    // stay in registers through the loop above.)
    if (sh.first[0]) {
        const auto *ab = argument_block();
        const int out_f32 = ab->d.out_f32;
        const u32x4 nan4 = out_f32 ? u32x4{0x7fc00000u, 0x7fc00000u, 0x7fc00000u, 0x7fc00000u}
                                   : u32x4{0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u};
        const int64_t rows = (int64_t)ab->d.B * ab->d.Hq;
        const int64_t out_quads = rows * D * (out_f32 ? 4 : 2) / 16;
        u32x4 *out4 = (u32x4 *)ab->d.out;
        for (int64_t i = threadIdx.x; i < out_quads; i += kThreads)
            out4[i] = nan4;
        float *lse = ab->d.lse, *part_lse = ab->d.part_lse;
        const int max_parts = ab->d.max_parts;
        if (lse)
            for (int64_t i = threadIdx.x; i < rows; i += kThreads)
                lse[i] = __builtin_nanf("");
        if (part_lse)
            for (int64_t i = threadIdx.x; i < rows * max_parts; i += kThreads)
                part_lse[i] = __builtin_nanf("");
    }
}

namespace {
// A launch without a caller's control area takes the next block of its half of the static pool,
// round robin.  A recorded launch keeps its block for every replay, which is why it must not
// share the pool with direct launches that may run beside a replay on another stream.
std::atomic<unsigned> g_next_slot{0}, g_next_recorded_slot{0};
}

bool decode_stream_supports(int d, int G, int B)
{
    (void)B; // any batch: more than kMaxStreamB rows go out as several launches
    return d == D && G >= 1 && G <= 16;
}

namespace {
struct DeviceInfo {
    uint32_t *pool = nullptr;        // g_pool
    uint32_t *pool_status = nullptr; // g_pool_status
    unsigned long long *faults = nullptr;
    int workgroups = 0;
};
DeviceInfo g_info[64];
std::atomic<int> g_ready[64];

// per-device set-up, once: addresses of the counters, LDS limit, grid size
hipError_t device_info(int *dev_out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    *dev_out = dev;
    if (g_ready[dev].load(std::memory_order_acquire))
        return hipSuccess;
    DeviceInfo di;
    if ((e = hipGetSymbolAddress((void **)&di.pool, HIP_SYMBOL(g_pool))) != hipSuccess)
        return e;
    if ((e = hipGetSymbolAddress((void **)&di.pool_status, HIP_SYMBOL(g_pool_status))) != hipSuccess)
        return e;
    if ((e = hipGetSymbolAddress((void **)&di.faults, HIP_SYMBOL(g_stream_faults))) != hipSuccess)
        return e;
    const void *kernels[] = {(const void *)decode_stream_kernel<false, 0>, (const void *)decode_stream_kernel<false, 4>,
                             (const void *)decode_stream_kernel<false, 3>,
                             (const void *)decode_stream_kernel<true, 0>, (const void *)decode_stream_kernel<true, 3>};
    for (const void *kernel : kernels)
        if ((e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes)) != hipSuccess)
            return e;
    int cus = 0;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess)
        return e;
    di.workgroups = cus; // compute units: a workgroup takes most, or half, of one's LDS
    g_info[dev] = di;
    g_ready[dev].store(1, std::memory_order_release);
    return hipSuccess;
}
} // namespace

namespace {
hipError_t launch_rows(const DecodeParams &p, int d, bool fp8, int chunk, hipStream_t stream);
}

// The kernel's length scan holds kMaxStreamB rows; a larger batch goes out as several launches
// over consecutive row ranges (each a full pass over its rows, into its own part of every
// per-row array).
hipError_t launch_decode_stream(const DecodeParams &p, int d, bool fp8, hipStream_t stream)
{
    if (!decode_stream_supports(d, p.G, p.B))
        return hipErrorInvalidValue;
    const size_t out_elem = p.out_f32 ? 4 : 2;
    for (int b0 = 0; b0 < p.B; b0 += kMaxStreamB) {
        DecodeParams c = p;
        c.B = std::min(kMaxStreamB, p.B - b0);
        c.q = p.q + (int64_t)b0 * p.q_row_stride;
        c.block_table = p.block_table + (int64_t)b0 * p.max_pages;
        c.seq_lens = p.seq_lens + b0;
        c.out = (char *)p.out + (size_t)b0 * p.Hq * D * out_elem;
        c.lse = p.lse ? p.lse + (int64_t)b0 * p.Hq : nullptr;
        c.part_o = p.part_o ? p.part_o + (int64_t)b0 * p.max_parts * p.Hq * D : nullptr;
        c.part_lse = p.part_lse ? p.part_lse + (int64_t)b0 * p.max_parts * p.Hq : nullptr;
        const hipError_t e = launch_rows(c, d, fp8, b0 / kMaxStreamB, stream);
        if (e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

namespace {
hipError_t launch_rows(const DecodeParams &p, int d, bool fp8, int chunk, hipStream_t stream)
{
    int dev = 0;
    hipError_t e = device_info(&dev);
    if (e != hipSuccess)
        return e;
    // LDS plan: the query tiles and the staging buffers of the group size are fixed costs, the
    // ring takes the rest.  bf16: one workgroup per compute unit, two staging buffers (one for
    // the widest groups).  fp8: a wave spends its time in the dependent chain of a step, not
    // waiting for memory, and its stages are half the size, so two workgroups share a compute
    // unit where they fit (measured: 1.3x; the depth of the ring hardly matters then: two stages
    // instead of three cost 3 %).  Groups of up to four heads fit three stages and both staging
    // buffers; wider ones give up the second staging buffer first (measured on ragged lengths: a
    // third stage is worth 3 to 9 % more than it).
    const int q_rows = (p.G + 3) / 4 * 4;
    const int stage_bytes = fp8 ? Geo<true>::kStage : Geo<false>::kStage;
    const int max_stages = fp8 ? Geo<true>::kMaxStages : Geo<false>::kMaxStages;
    auto fixed_bytes = [&](int staging_buffers) {
        return sizeof(Shared) + (size_t)kWaves * q_rows * (D * 2) +
               (size_t)staging_buffers * kWaves * p.G * D * sizeof(float);
    };
    auto stages_for = [&](int workgroups_per_cu, int staging_buffers) {
        const size_t share = (size_t)kMaxLdsBytes / workgroups_per_cu, fixed = fixed_bytes(staging_buffers);
        return share > fixed ? std::min((int)((share - fixed) / ((size_t)kWaves * stage_bytes)), max_stages) : 0;
    };
    const int nb_default = p.G > 8 ? 1 : 2;
    int per_cu = 1, nb = nb_default, stages = 0;
    if (fp8 && stages_for(2, nb_default) >= 3) {
        per_cu = 2;
    } else if (fp8 && stages_for(2, 1) >= 3) {
        per_cu = 2;
        nb = 1;
    } else if (fp8 && stages_for(2, nb_default) >= 2) {
        per_cu = 2;
    }
    stages = stages_for(per_cu, nb);
    if (stages < 2)
        return hipErrorInvalidValue;
    const size_t fixed = fixed_bytes(nb);
    const size_t lds = (size_t)kWaves * stages * stage_bytes + fixed;
    StreamParams sp;
    sp.d = p;
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capturing) != hipSuccess)
        (void)hipGetLastError();
    if (p.control) { // the caller's control area: status block, then one block per launch of the call
        sp.status = p.control;
        sp.ctl = p.control + (size_t)(1 + chunk) * kControlBlockWords;
    } else {
        const unsigned slot = capturing == hipStreamCaptureStatusNone
                                  ? g_next_slot.fetch_add(1) % (kTicketSlots / 2)
                                  : kTicketSlots / 2 + g_next_recorded_slot.fetch_add(1) % (kTicketSlots / 2);
        sp.status = g_info[dev].pool_status;
        sp.ctl = g_info[dev].pool + 4 * slot;
    }
    sp.faults = g_info[dev].faults;
    sp.pt = p.partition_tokens > 0 ? p.partition_tokens : (1 << 30);
    sp.stages = stages;
    sp.nb = nb;
    sp.q_rows = q_rows;
    // A stream may be confined to some of the compute units: size the grid for those.
    // (Not asked of a stream that is recording a graph: queries can end a capture.)
    int cus = g_info[dev].workgroups;
    if (p.grid_cus > 0) {
        cus = std::min(cus, p.grid_cus);
    } else if (capturing == hipStreamCaptureStatusNone) {
        uint32_t mask[32] = {0};
        if (hipExtStreamGetCUMask(stream, 32, mask) == hipSuccess) {
            int bits = 0;
            for (uint32_t w : mask)
                bits += __builtin_popcount(w);
            if (bits > 0 && bits < cus)
                cus = bits;
        } else {
            (void)hipGetLastError(); // not an error of this call's work
        }
    }
    int64_t grid = (int64_t)p.B * p.Hkv * p.max_parts;
    if (grid > (int64_t)cus * per_cu)
        grid = (int64_t)cus * per_cu;
    const dim3 blocks((unsigned)grid);
    const bool fixed_depth = p.page_shift == 0;
    if (fp8 && stages == 3 && fixed_depth)
        decode_stream_kernel<true, 3><<<blocks, kThreads, lds, stream>>>(sp);
    else if (fp8)
        decode_stream_kernel<true, 0><<<blocks, kThreads, lds, stream>>>(sp);
    else if (stages == 4 && fixed_depth)
        decode_stream_kernel<false, 4><<<blocks, kThreads, lds, stream>>>(sp);
    else if (stages == 3 && fixed_depth) // groups of five to eight heads
        decode_stream_kernel<false, 3><<<blocks, kThreads, lds, stream>>>(sp);
    else
        decode_stream_kernel<false, 0><<<blocks, kThreads, lds, stream>>>(sp);
    return hipGetLastError();
}
} // namespace

// Number of bounded waits that expired in any launch on the current device since
// the library was loaded (0 unless the kernel's hand-shakes are broken).  Synchronises.
hipError_t read_stream_faults(unsigned long long *count)
{
    int dev = 0;
    hipError_t e = device_info(&dev);
    if (e != hipSuccess)
        return e;
    return hipMemcpy(count, g_info[dev].faults, sizeof(*count), hipMemcpyDeviceToHost);
}

} // namespace adr
