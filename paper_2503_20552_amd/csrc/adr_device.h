// Device-side helpers and kernel parameter blocks shared by the gfx950 kernels.
// Wave size is 64 everywhere in this library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adr {

constexpr int kPageSize = 16;       // tokens per tile, the kernels' unit of work: a cache page of 16 << page_shift
                                    // tokens is 1 << page_shift consecutive tiles of the pool
constexpr int kWaves = 4;           // waves per workgroup in the attention kernels
constexpr int kThreads = kWaves * 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f; // "no score seen yet": finite so that differences never give NaN
constexpr int kSpinLimit = 1 << 24; // polls of a flag in on-chip memory before a wait on another wave is declared
                                    // failed (seconds: an unsplit row of millions of tokens keeps a wave busy for
                                    // tens of ms)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

// Control area of a call, in the caller's workspace behind the partial results (or, for a call
// without a workspace, in a small static pool): one block of call status, then one block per
// launch of the resident-workgroup kernel (a batch goes out as one launch per 512 rows).
// Every word is zero when no launch is using the area: an initialising kernel (or the append
// kernel of adr_decode_step) clears it, and each launch hands its own block back cleared.
constexpr int kControlBlockBytes = 256;
constexpr int kControlBlockWords = kControlBlockBytes / 4;
enum {
    kStatusExpiredWaits = 0, // call status, word 0: bounded waits that expired since the area was cleared
    kLaunchTicket = 0,       // launch block: next ticket
    kLaunchFinished = 1,     //   workgroups that are through
    kLaunchExpired = 2,      //   bounded waits that expired in this launch
};

// What a debug build (-DADR_DEBUG_BOUNDS) records about table entries and positions that fall
// outside the pool or the table: how many, and the first one.
struct BoundsRecord {
    uint32_t count;
    int32_t kind; // 0 none, 1 attention: page id outside the pool, 2 append: position outside the table,
                  // 3 append: page id outside the pool
    int32_t row, index, value;
};

// Everything adr_decode_attention's kernels need, passed by value.
struct DecodeParams {
    const uint16_t *q;
    int64_t q_row_stride; // elements between request rows of q
    const void *k_cache, *v_cache;
    const float *k_scale, *v_scale;
    const int32_t *block_table;
    const int32_t *seq_lens;
    void *out;       // [B][Hq][d] bf16 or fp32
    float *lse;      // [B][Hq] or nullptr
    float *part_o;   // [B][max_parts][Hq][d] normalised partial outputs (split pass)
    float *part_lse; // [B][max_parts][Hq] natural-log lse of each partition
    int max_pages;   // row length of block_table
    int page_shift;  // log2(page_size / 16)
    int B, Hq, Hkv, G, num_pages;
    int partition_tokens; // 0 = whole sequence in one pass
    int max_parts;        // partitions per request the grid was sized for (>= 1)
    int max_seq_len;
    int out_f32;          // 1: out is fp32, 0: bf16
    int coalesce;         // the resident kernel may take runs of partitions as one item
    float scale_log2e;    // softmax scale * log2(e): scores are kept in base 2
    uint32_t *control;    // control area of the call (status block first), or nullptr: the static pool
    int spin_limit;       // polls before a wait on another wave is declared failed
    int grid_cus;         // > 0: size the resident kernel's grid for this many compute units
    BoundsRecord *bounds; // debug builds: where out-of-range entries are recorded (else nullptr)
};

struct MergeParams {
    void *out;
    float *lse_out;
    const float *part_o, *part_lse;
    const int32_t *part_offsets; // CSR [B+1], or nullptr for the implicit layout below
    const int32_t *seq_lens;     // implicit layout: request b owns partitions
    int partition_tokens;        //   [b*max_parts, b*max_parts + ceil(min(seq_len,max_seq_len)/partition_tokens))
    int max_parts, max_seq_len;  //   and rows with <= 1 partition are left alone
    int B, heads, d, out_f32;
    const uint32_t *status;      // call status block of the pass that wrote the partials, or nullptr: when
                                 // its expired-waits word is not zero every row gets NaN
};

struct AppendParams {
    void *k_cache, *v_cache;
    float *k_scale, *v_scale;
    const uint16_t *k_new, *v_new;
    int64_t new_row_stride; // elements between request rows of k_new / v_new
    const int32_t *block_table, *positions;
    // positions == nullptr: the token index is min(max(seq_lens[b], 0), max_seq_len) - 1
    // (the last token of the row as the attention kernels see it; an empty row is skipped)
    const int32_t *seq_lens;
    int max_seq_len;
    int max_pages, num_pages, page_size, Hkv, d, B;
    uint32_t *clear_words; // control area the first workgroup clears on its way (adr_decode_step), or nullptr
    int n_clear_words;
    BoundsRecord *bounds;  // debug builds only
};

// positions == nullptr: the row's last token as the attention kernels will see it.  A row
// longer than the host's bound is attended up to the bound and appends nothing: writing at the
// bound would overwrite an older token.
__device__ __forceinline__ int append_position(const AppendParams &p, int b)
{
    if (p.positions)
        return p.positions[b];
    const int L = p.seq_lens[b];
    return L > p.max_seq_len ? -1 : L - 1;
}

__device__ __forceinline__ void record_out_of_bounds(BoundsRecord *rec, int kind, int row, int index, int value)
{
#ifdef ADR_DEBUG_BOUNDS
    if (rec) {
        atomicAdd(&rec->count, 1u);
        if (atomicCAS(&rec->kind, 0, kind) == 0) {
            rec->row = row;
            rec->index = index;
            rec->value = value;
        }
    }
#else
    (void)rec; (void)kind; (void)row; (void)index; (void)value;
#endif
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Cross-lane moves inside a row of 16 lanes (DPP, no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), CTRL, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16 lanes

// Sum over aligned groups of LANES lanes (LANES = 8 or 16); every lane of the
// group ends with the group's total.
template <int LANES>
__device__ __forceinline__ float group_sum(float x)
{
    x += dpp_mov<kDppXor1>(x);
    x += dpp_mov<kDppXor2>(x);
    x += dpp_mov<kDppHalfMirror>(x); // quads hold equal values, so the mirror acts as xor 4
    if (LANES == 16)
        x += dpp_mov<kDppMirror>(x);
    return x;
}

// Reductions over the four lanes l, l^16, l^32, l^48 (the four 16-lane rows of a wave) with the
// row-swap instructions of gfx950: v_permlane16_swap exchanges the odd rows of its first operand
// with the even rows of its second, v_permlane32_swap the upper half of the first with the lower
// half of the second.  Fed the same value twice, the two results hold, in every lane, the lane's
// own value and its partner's (in one order or the other), so a commutative operation of the two
// is the pairwise reduction.  No LDS traffic, unlike a lane shuffle.
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ float max_across_rows(float x)
{
    u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float sum_across_rows(float x)
{
    u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
#else // the host pass only parses device code
__device__ __forceinline__ float max_across_rows(float x) { return x; }
__device__ __forceinline__ float sum_across_rows(float x) { return x; }
#endif

__device__ __forceinline__ int clamp_page(int page, int num_pages)
{
    return min(max(page, 0), num_pages - 1);
}

// Tile `tile` of a row, as an index among all 16-token tiles of the pool: the row's table entry
// for the page the tile lies in (clamped into the pool), times the tiles of a page, plus the
// tile's place in its page.
__device__ __forceinline__ int pool_tile(int table_entry, int tile, int num_pages, int page_shift)
{
    return (clamp_page(table_entry, num_pages) << page_shift) | (tile & ((1 << page_shift) - 1));
}

// The same, for kernels that know which row they are in: a debug build records an entry that
// had to be clamped (the release build clamps silently).
__device__ __forceinline__ int pool_tile_checked(int table_entry, int tile, int num_pages, int page_shift,
                                                 BoundsRecord *rec, int row)
{
#ifdef ADR_DEBUG_BOUNDS
    if ((unsigned)table_entry >= (unsigned)num_pages && (threadIdx.x & 63) == 0)
        record_out_of_bounds(rec, 1, row, tile >> page_shift, table_entry);
#else
    (void)rec; (void)row;
#endif
    return pool_tile(table_entry, tile, num_pages, page_shift);
}

// Number of partitions of a row of L tokens (>= 1, so that an empty row still
// owns the partition that writes its zeros).
__device__ __forceinline__ int parts_of(int L, int partition_tokens)
{
    if (partition_tokens <= 0 || L <= 0)
        return 1;
    return (L + partition_tokens - 1) / partition_tokens;
}

// Combine the kWaves per-wave partial results staged in LDS and write either
// the final output row or this partition's (normalised o, lse) pair.
// sm/sl: [kWaves][G] running max (base 2) and denominator; so: [kWaves][G][D].
template <int D>
__device__ __forceinline__ void combine_waves_and_store(const DecodeParams &p, const float *sm,
                                                        const float *sl, const float *so, int G,
                                                        int b, int kvh, int part, int n_parts)
{
    for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
        const int g = idx / D, dd = idx - g * D;
        float M = sm[g];
#pragma unroll
        for (int w = 1; w < kWaves; ++w)
            M = fmaxf(M, sm[w * G + g]);
        float acc = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float f = fast_exp2(sm[w * G + g] - M);
            acc += f * so[(w * G + g) * D + dd];
            den += f * sl[w * G + g];
        }
        const float o = den > 0.f ? acc / den : 0.f;
        const float lse = den > 0.f ? (M + fast_log2(den)) * kLn2 : -INFINITY;
        const int h = kvh * G + g;
        if (n_parts == 1) {
            const int64_t off = ((int64_t)b * p.Hq + h) * D + dd;
            if (p.out_f32)
                ((float *)p.out)[off] = o;
            else
                ((uint16_t *)p.out)[off] = (uint16_t)f32_to_bf16(o);
            if (p.lse && dd == 0)
                p.lse[(int64_t)b * p.Hq + h] = lse;
        } else {
            const int64_t row = ((int64_t)b * p.max_parts + part) * p.Hq + h;
            p.part_o[row * D + dd] = o;
            if (dd == 0)
                p.part_lse[row] = lse;
        }
    }
}

} // namespace adr
