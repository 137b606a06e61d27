/*
 * adr.h -- C ABI of the MI355X (gfx950) paged decode-attention library.
 *
 * The library implements the per-layer work of the paper's attention executor
 * (Sec. 3.1 "Overview": an executor colocated with the prefill engine runs the
 * decode-phase attention that was offloaded to it; Sec. 3.2.1: per layer it
 * receives the grouped q,k,v of the offloaded requests, runs the attention
 * kernel over its own KV cache kept in cache blocks with per-request metadata,
 * and returns the attention output).  The operation itself is step (2) of a
 * transformer layer in Sec. 2.1: attention of the decode step's single query
 * token per head over the request's cached K and V, after the new token's K
 * and V have been added to the cache.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers, borrowed for the duration of the
 *    enqueued work; the library never allocates, frees or retains memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue kernels: no synchronisation, no allocation, no copies
 *    to the host, grids sized from host scalars only, so a call may be recorded
 *    into a HIP graph (Sec. 3.2.2 relies on replaying pre-launched kernels).
 *  - Concurrency: calls on different streams of one device may overlap as long as they do not
 *    share a workspace (two calls, or two replays of one recorded graph, that use one workspace
 *    at the same time race on its contents).  The counters the attention kernels hand work out
 *    with live in the workspace.  Only a call WITHOUT a workspace (an unsplit pass, workspace
 *    NULL) falls back on a pool of 128 + 128 counter blocks inside the library (direct launches
 *    and launches recorded into graphs); more than 128 such launches running at once, or 128
 *    such recorded launches alive at once, would share blocks: give such calls the (small)
 *    workspace adr_decode_workspace_bytes reports for partition_tokens = 0 instead.
 *  - Return value: ADR_OK or an error code.  Every host-checkable violation is
 *    reported BEFORE anything is launched and leaves all buffers untouched.
 *  - bf16 = upper 16 bits of IEEE binary32.  fp8 = OCP E4M3 (finite-only
 *    variant: bias 7, max 448, S.1111.111 = NaN).
 *  - Supported set: d in {64, 128}; page_size in {16, 32, 64}; Hq a multiple of Hkv with
 *    G = Hq/Hkv <= 16; cache dtype bf16 or fp8-e4m3; output bf16 or fp32.
 *    q-head h reads kv-head h / G.
 *  - Alignment: q, k_new, v_new, the caches and `out` must be 16-byte aligned
 *    and row strides must keep every row 16-byte aligned.
 */
#ifndef ADR_H
#define ADR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ADR_OK = 0,
    ADR_ERR_NULL = 1,        /* a required pointer is NULL */
    ADR_ERR_SHAPE = 2,       /* a size is non-positive, inconsistent or misaligned */
    ADR_ERR_UNSUPPORTED = 3, /* outside the supported set above */
    ADR_ERR_WORKSPACE = 4,   /* split pass requested but workspace missing / too small */
    ADR_ERR_LAUNCH = 5       /* the HIP runtime refused a launch */
} adr_status;

typedef enum { ADR_BF16 = 0, ADR_FP8_E4M3 = 1, ADR_F32 = 2 } adr_dtype;

/* Kernel choice for adr_decode_attention (bits 0..3 of `flags`). */
enum {
    ADR_KERNEL_AUTO = 0, /* the library picks per shape */
    ADR_KERNEL_VALU = 1, /* vector-ALU dot products: d in {64, 128}, G in {1, 2, 4, 8} */
    ADR_KERNEL_MFMA = 2, /* matrix-core QK^T and PV (d = 128): resident workgroups pulling
                            (request, partition, kv-head) items; batches of more than 512 rows
                            go out as one launch per 512 rows */
    ADR_KERNEL_MFMA_GRID = 3, /* matrix cores, one workgroup per (request, partition, kv-head), for up
                                 to 33 partitions of a request (workgroups loop over the partitions
                                 of longer ones); its grid is sized from max_seq_len, so a bound far
                                 above the lengths costs it time; bf16 cache only */
    /* Bit 4: run the partition pass only and leave the merge to a later
     * adr_decode_merge call on the same workspace (rows with one partition are
     * still written to `out` directly).  Lets a caller place the two passes on
     * a stream itself, e.g. to time them separately. */
    ADR_PARTIALS_ONLY = 16,
    /* Every partition is attended as an item of its own.  Without this flag the resident
     * matrix-core kernel, when a pass has many thousands of partitions, takes runs of two or
     * four neighbouring partitions of a row as one item: the run's result stands in the
     * workspace at its first partition's place and the others are marked empty (lse = -inf),
     * which the merge skips.  The final result is the same up to the order of the
     * floating-point sums; the choice depends on the inputs alone. */
    ADR_SINGLE_PARTITION_ITEMS = 32,
    /* The caller vouches that the workspace's control area (its last bytes, see
     * adr_decode_workspace_bytes) is all zero: it was cleared by an earlier call on this workspace
     * that has completed, and every call leaves it zero.  Saves adr_decode_attention the small
     * kernel that clears it first (adr_decode_step never needs one).  On an area that is not zero
     * the results are wrong or NaN. */
    ADR_WORKSPACE_READY = 64,
    /* Test aid: the resident matrix-core kernel's waits on other waves expire at once, as if its
     * hand-shakes were broken.  Every kernel still runs to its end; the call's rows come back as
     * NaN and adr_decode_read_status reports the expired waits. */
    ADR_DEBUG_EXPIRE_WAITS = 128
};
/* Bits 16..27 of `flags`: size the resident kernel's grid for n compute units (1..4095) instead
 * of asking the stream for its compute-unit mask.  Needed while a graph is being recorded for a
 * masked stream: a recording stream cannot be asked, and the grid is then sized for the whole
 * chip. */
#define ADR_GRID_CUS(n) (((unsigned)(n) & 0xFFFu) << 16)

/* The paged KV cache of ONE layer ("cache blocks", Sec. 3.2.1).  K and V are
 * separate arrays of identical shape [num_pages][page_size][Hkv][d],
 * contiguous.  Token t of a request lives in page block_table[b][t/page_size],
 * slot t % page_size.  For fp8 caches each (page, kv-head) has one fp32 scale,
 * separately for K and V: value = decode(byte) * scale. */
typedef struct adr_kv_cache {
    void *k, *v;
    float *k_scale, *v_scale; /* [num_pages][Hkv]; NULL unless dtype == ADR_FP8_E4M3 */
    int num_pages, page_size, Hkv, d;
    adr_dtype dtype;
} adr_kv_cache;

/*
 * adr_kv_append -- store the decode step's new token (Sec. 2.1: the decode
 * phase computes K and V only for the new token; they join the cache).
 *
 *   k_new, v_new  bf16 [B][Hkv][d]; request rows `new_row_stride` ELEMENTS
 *                 apart (so both may be views into one grouped q|k|v buffer,
 *                 Sec. 3.2.1 step 2); heads and d contiguous.
 *   block_table   int32 [B][max_pages_per_req], physical page ids.
 *   positions     int32 [B]: token index to write = request length before the
 *                 append; negative = skip this row (a padded batch row).
 *
 * bf16 cache: a bit-for-bit copy.  fp8 cache: the token landing in slot 0 of a
 * page sets that page's scale to 2*amax(|x| over d, floored at 2^-20)/448 per
 * kv-head; every token is stored as round-to-nearest-even, saturating
 * E4M3(x * (1/scale)) computed in fp32.
 * A position outside the row's table, or a page id outside [0,num_pages), makes
 * the kernel skip that row (nothing written); it is not reported.
 * Two rows naming the same (page, slot) race.
 */
int adr_kv_append(const adr_kv_cache *cache, const void *k_new, const void *v_new,
                  int64_t new_row_stride, const int32_t *block_table, int max_pages_per_req,
                  const int32_t *positions, int B, void *stream);

/* Bytes of workspace for a call of adr_decode_attention / adr_decode_step; depends only on host
 * scalars (0 for sizes that are not positive).  The workspace holds the partitions' results of a
 * split pass (nothing when partition_tokens == 0) and, in its last 256 * (1 + ceil(B / 512))
 * bytes, the call's control area: a status block and the counters the resident kernel hands
 * work out with.  A split pass needs the workspace; an unsplit one may do without (see
 * "Concurrency" above).  The contents need no initialisation by the caller. */
size_t adr_decode_workspace_bytes(int B, int Hq, int d, int max_seq_len, int partition_tokens);

/*
 * adr_decode_attention -- for every request b and q-head h:
 *     out[b][h][:] = sum_t softmax_t(scale * <q[b][h], K_t>) * V_t,
 * t over the first seq_lens[b] cached tokens of request b, K_t/V_t taken from
 * kv-head h/G (Sec. 2.1 step (2); the kernel the executor of Sec. 3.1 runs).
 *
 *   out        [B][Hq][d], bf16 or fp32 (out_dtype), contiguous.
 *   lse        optional fp32 [B][Hq]: natural-log log-sum-exp of the scaled scores.
 *   q          bf16 [B][Hq][d], request rows q_row_stride ELEMENTS apart.
 *   seq_lens   int32 [B]: tokens attended (the length AFTER the append, so the
 *              new token attends to itself).  0 = padded row: out row = 0,
 *              lse = -inf, no cache memory is read.
 *   max_seq_len  host-side upper bound on seq_lens (sizes the grid; a row whose
 *              seq_len exceeds it is truncated to it).
 *   partition_tokens  0: one pass per (request, kv-head).  Otherwise a multiple
 *              of page_size: the sequence is cut into partitions of that many
 *              tokens, attended independently, and merged by log-sum-exp; needs
 *              `workspace` of adr_decode_workspace_bytes(...) bytes (256-byte
 *              aligned).  Rows with a single partition bypass the merge.
 *   flags      ADR_KERNEL_* in bits 0..3, optionally | ADR_PARTIALS_ONLY |
 *              ADR_SINGLE_PARTITION_ITEMS; other bits must be 0.
 *
 * Page ids are clamped into [0,num_pages) before use; table entries past
 * ceil(seq_len/page_size) are never dereferenced.  Results are bit-identical
 * from run to run for fixed inputs, partition_tokens and flags, and do not
 * depend on where pages sit in the pool.
 */
int adr_decode_attention(void *out, adr_dtype out_dtype, float *lse, const void *q,
                         int64_t q_row_stride, const adr_kv_cache *cache,
                         const int32_t *block_table, int max_pages_per_req,
                         const int32_t *seq_lens, int B, int Hq, float scale, int max_seq_len,
                         int partition_tokens, void *workspace, size_t workspace_bytes,
                         unsigned flags, void *stream);

/*
 * adr_decode_attention_static -- adr_decode_attention for callers that cannot allocate device
 * memory and have no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, checks and results as adr_decode_attention
 * (the same kernels run); the workspace (partitions' results and the control area) is a static
 * device array inside the library, ADR_STATIC_SCRATCH_BYTES long, which every device the library
 * runs on holds until the process ends.  The call itself allocates and frees nothing.
 *   - ADR_ERR_WORKSPACE when adr_decode_workspace_bytes(B, Hq, d, max_seq_len, partition_tokens)
 *     exceeds ADR_STATIC_SCRATCH_BYTES (B = 256, Hq = 32, d = 128, 8192-token rows in partitions
 *     of 512 need 68.6 MiB).  ADR_WORKSPACE_READY is refused (ADR_ERR_UNSUPPORTED).
 *   - Every call on a device uses that device's one array: calls that overlap on one device
 *     (two streams, or a replay beside a direct call) race on it.  The array keeps the last
 *     call's contents; each call clears what it needs cleared (the control area) with a small
 *     kernel of its own.
 */
#define ADR_STATIC_SCRATCH_BYTES (96u << 20)
int adr_decode_attention_static(void *out, adr_dtype out_dtype, float *lse, const void *q, int64_t q_row_stride,
                                const adr_kv_cache *cache, const int32_t *block_table, int max_pages_per_req,
                                const int32_t *seq_lens, int B, int Hq, float scale, int max_seq_len,
                                int partition_tokens, unsigned flags, void *stream);

/*
 * adr_decode_step -- one decode step of the executor (Sec. 2.1 steps (1)-(2), Sec. 3.2.1): the
 * new token's K/V join the cache and the row attends over all its tokens, the new one included.
 * Same result, in `out`, `lse` and the cache, as
 *     adr_kv_append(cache, k_new, v_new, new_row_stride, block_table, max_pages_per_req, pos, B, stream)
 *     with pos[b] = seq_lens[b] - 1, or -1 (append nothing) for an empty row and for a row with
 *     seq_lens[b] > max_seq_len: such a row is attended up to the bound, where an older token sits,
 * followed by adr_decode_attention with the remaining arguments.
 *
 *   k_new, v_new  bf16 [B][Hkv][d], rows new_row_stride ELEMENTS apart (views into the grouped
 *                 q|k|v buffer are fine), 16-byte aligned; read only.
 *   everything else as in adr_decode_attention; seq_lens is the length AFTER the append.
 *
 * The append kernel runs first, then the attention kernels, all on `stream`; the call saves the
 * caller the positions array (it is seq_lens - 1) and one trip through the binding.  k_new /
 * v_new must not alias the cache.
 */
int adr_decode_step(void *out, adr_dtype out_dtype, float *lse, const void *q, int64_t q_row_stride,
                    const void *k_new, const void *v_new, int64_t new_row_stride,
                    const adr_kv_cache *cache, const int32_t *block_table, int max_pages_per_req,
                    const int32_t *seq_lens, int B, int Hq, float scale, int max_seq_len,
                    int partition_tokens, void *workspace, size_t workspace_bytes, unsigned flags,
                    void *stream);

/*
 * adr_decode_merge -- the second pass of a split adr_decode_attention that was
 * called with ADR_PARTIALS_ONLY: merges the partitions left in `workspace` into
 * out / lse for every row with more than one partition; other rows are left as
 * the first pass wrote them.  B, Hq, d, seq_lens, max_seq_len, partition_tokens
 * and the workspace must be those of the first pass (partition_tokens is checked to be a
 * multiple of 16 only; the first pass also held it to the cache's page size).  A no-op
 * (ADR_OK) when the first pass did not split (max_seq_len <= partition_tokens or
 * partition_tokens == 0).  If the first pass reported expired waits in the workspace's status
 * block, every row of out / lse is set to NaN.
 */
int adr_decode_merge(void *out, adr_dtype out_dtype, float *lse, const int32_t *seq_lens, int B,
                     int Hq, int d, int max_seq_len, int partition_tokens, const void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * adr_lse_merge -- combine attention results computed over disjoint token sets
 * of the same request (the split pass of adr_decode_attention uses it; the
 * same pair (o, lse) is what a second device would ship for a sequence-sharded
 * request):
 *     lse*  = ln sum_p exp(part_lse[p][h])
 *     out[b][h][:] = sum_p exp(part_lse[p][h] - lse*) * part_o[p][h][:]
 *
 *   part_o       fp32 [total_parts][heads][d], each already normalised by its
 *                own softmax denominator.
 *   part_lse     fp32 [total_parts][heads], natural log; -inf = empty partition
 *                (its part_o is ignored, even if NaN).
 *   part_offsets int32 [B+1]: request b owns partitions [off[b], off[b+1]).
 *   out          [B][heads][d] bf16 or fp32; lse_out optional fp32 [B][heads].
 * A request with no partitions, or only empty ones, gives zeros and -inf.
 */
int adr_lse_merge(void *out, adr_dtype out_dtype, float *lse_out, const float *part_o,
                  const float *part_lse, const int32_t *part_offsets, int B, int heads, int d,
                  void *stream);

/*
 * Measurement aids (not part of the attention path): a streaming read of
 * `bytes` bytes (multiple of 16) that folds everything into 4 bytes per
 * workgroup written to `sink` (>= 64 KiB), and a plain copy.  They give the
 * box's attainable HBM rate and calibrate the profiler's byte counters.
 */
int adr_probe_stream_read(const void *src, size_t bytes, void *sink, void *stream);
int adr_probe_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Streams confined to a subset of the compute units (Sec. 3.3: the executor and
 * the prefill engine share one GPU, each on a fraction of its cores; the paper
 * sets the split with MPS, here it is a queue's compute-unit mask).
 * adr_stream_create_cu_mask returns in *stream (a HOST pointer to a void*) a new
 * hipStream_t of default priority whose kernels run only on the compute units
 * whose bit is set in cu_mask (HOST pointer, n_words 32-bit words, bit i of word
 * w = unit 32*w + i); pass it as `stream` to the calls above, or wrap it for
 * other libraries.  adr_stream_destroy releases it after its work has finished.
 * Errors: ADR_ERR_NULL, ADR_ERR_SHAPE (n_words <= 0 or an empty mask),
 * ADR_ERR_LAUNCH (the runtime refused).
 */
int adr_stream_create_cu_mask(void **stream, const uint32_t *cu_mask, int n_words);
int adr_stream_destroy(void *stream);

/*
 * Copies around the attention call (decode side of Sec. 3.2.1 / 3.2.2); bf16, bit for bit, 16-byte
 * pieces: d and every row stride (in ELEMENTS) must be multiples of 8, pointers 16-byte aligned.
 *
 * adr_pack_qkv -- "grouping qkv": dst[b] = q[b] | k[b] | v[b], i.e. Hq*d, Hkv*d and Hkv*d elements
 *   side by side in a row of dst (row stride >= (Hq + 2 Hkv) * d), so that the three tensors travel
 *   as one message and the receiver passes views of that buffer to adr_kv_append and
 *   adr_decode_attention.  q, k, v: [B][heads][d] with their own row strides.
 * adr_scatter_rows -- "merging outputs": dst[row_index[i]][0..row_elems) = src[i][0..row_elems) for
 *   i < n_rows: the rows an executor returned take their places among the rows of the decode
 *   batch's output (dst has dst_rows rows).  row_index is a DEVICE int32 array; an index outside
 *   [0, dst_rows) skips that row; equal indices race.
 */
int adr_pack_qkv(void *dst, int64_t dst_row_stride, const void *q, int64_t q_row_stride, const void *k,
                 int64_t k_row_stride, const void *v, int64_t v_row_stride, int B, int Hq, int Hkv, int d,
                 void *stream);
int adr_scatter_rows(void *dst, int64_t dst_row_stride, int dst_rows, const void *src, int64_t src_row_stride,
                     const int32_t *row_index, int n_rows, int row_elems, void *stream);

/*
 * Host-side arithmetic of the paper's proxy (no device work, no stream).
 *
 * Offloading-ratio bound, Sec. 3.4.1:
 *   adr_offload_bound_mem   Eq. 1: min(sum_i HBM_p[i] / HBM_d, sum_i BW_p[i] / BW_d) over the n
 *                           prefill instances serving one decode instance (HOST arrays of n
 *                           values, any consistent unit).  NaN when a denominator is not positive
 *                           or an array is missing.
 *   adr_offload_bound_comp  Eq. 2: (B_max - B_TPOT) / B_TPOT.  NaN when B_TPOT is not positive.
 *   adr_offload_bound       Eq. 3: the smaller of the two.
 * adr_need_offload, Algorithm 1 (Sec. 3.4.3): 1 when the new request's attention may be offloaded,
 *   0 when not, and -ADR_ERR_NULL (a negative number: compare the result with 1, do not test it
 *   as a boolean) on a missing array.  `local` / `offloaded` are the decode
 *   instance's running and offloaded requests; a request is its maximal and its current token
 *   count.  Read as printed: both conditions compare with strict "<", and the sum of the offloaded
 *   requests' maximal lengths, which the listing computes, enters neither condition.
 * adr_graph_capacity, Sec. 3.2.2: the smallest multiple of `interval` that is >= n (at least one
 *   interval) if it does not exceed max_capacity, else -1: the recorded graph a batch of n rows is
 *   replayed with, the other rows being padded rows (seq_len 0, position < 0).
 */
typedef struct adr_request_tokens {
    int64_t max_token;  /* prompt plus the most it may generate */
    int64_t used_token; /* tokens it holds now */
} adr_request_tokens;

double adr_offload_bound_mem(const double *hbm_prefill, const double *bw_prefill, int n, double hbm_decode,
                             double bw_decode);
double adr_offload_bound_comp(double b_max, double b_tpot);
double adr_offload_bound(double ob_mem, double ob_comp);
int adr_need_offload(const adr_request_tokens *req, const adr_request_tokens *local, int n_local,
                     const adr_request_tokens *offloaded, int n_offloaded, double bound);
int adr_graph_capacity(int n, int interval, int max_capacity);

/*
 * Table of pre-recorded decode steps (Sec. 3.2.2, "Kernel Pre-launching": the executor's kernels
 * are launched from recorded graphs, because launching them one by one costs more CPU time than
 * they take on the GPU; graphs exist for batch capacities on an interval grid and a batch replays
 * the smallest one that holds it).
 *
 * adr_graph_table_create records, for every capacity interval, 2*interval, ..., max_capacity (a
 * multiple of interval), one step of that many rows -- adr_decode_step for each of the n_layers
 * caches in turn, on the buffers described by *buffers -- from capture_stream (a stream other than
 * the default one, idle, which the call leaves idle), and instantiates the graphs.  The buffers must
 * hold max_capacity rows and outlive the table; `caches` is a HOST array that is only read during
 * the call.  This call allocates (graphs); launching does not.
 * adr_graph_table_launch replays, on `stream`, the smallest recorded capacity >= n_rows
 * (ADR_ERR_SHAPE if there is none).  Before each launch the caller writes the step's inputs into
 * the buffers; rows from n_rows up to that capacity must be padded rows (seq_lens 0), which append
 * nothing, read no cache memory and get a zero output row.  Replays of one table must not overlap
 * each other (they share the buffers and the workspace).
 * adr_graph_table_capacity: the capacity a batch of n_rows would replay, or -1.
 * A table for a stream confined to some compute units is recorded with ADR_GRID_CUS(n) in
 * buffers->flags and launched on that stream: the recording stream cannot be asked for its mask.
 */
typedef struct adr_step_buffers {
    void *out;              /* [max_capacity][Hq][d] */
    adr_dtype out_dtype;
    float *lse;             /* optional [max_capacity][Hq] */
    const void *q;          /* bf16 [max_capacity][Hq][d], rows q_row_stride elements apart */
    int64_t q_row_stride;
    const void *k_new, *v_new; /* bf16 [max_capacity][Hkv][d], rows new_row_stride elements apart */
    int64_t new_row_stride;
    const adr_kv_cache *caches; /* HOST array: the layers' caches, attended in this order */
    int n_layers;
    const int32_t *block_table; /* [max_capacity][max_pages_per_req] */
    int max_pages_per_req;
    const int32_t *seq_lens;    /* [max_capacity]: lengths after the append; 0 = padded row */
    int Hq;
    float scale;
    int max_seq_len, partition_tokens;
    void *workspace;            /* adr_decode_workspace_bytes(max_capacity, ...) bytes */
    size_t workspace_bytes;
    unsigned flags;
} adr_step_buffers;
typedef struct adr_graph_table adr_graph_table;
int adr_graph_table_create(adr_graph_table **table, const adr_step_buffers *buffers, int interval,
                           int max_capacity, void *capture_stream);
int adr_graph_table_capacity(const adr_graph_table *table, int n_rows);
int adr_graph_table_launch(adr_graph_table *table, int n_rows, void *stream);
int adr_graph_table_destroy(adr_graph_table *table);

/*
 * Self-check of the resident-workgroup kernel (ADR_KERNEL_MFMA): its waves hand
 * work to each other through flags in on-chip memory, and every wait on such a
 * flag is bounded.  When one expires the kernel still runs to its end, but no row of
 * that launch can be trusted: the launch's rows of out / lse (and its partitions' lse)
 * are overwritten with NaN, the merge of a split pass sets every row of the call to NaN,
 * and the expiry is counted in the workspace's status block and device-wide.
 *   adr_decode_read_status  `*expired_waits` (HOST pointer) receives the status block's count
 *       of the workspace (same B, Hq, d, max_seq_len, partition_tokens as the call): waits that
 *       expired in calls on it since its control area was last cleared (every call clears it
 *       unless it passes ADR_WORKSPACE_READY).  ADR_ERR_WORKSPACE when there is none.
 *   adr_stream_fault_count  `*count` (HOST pointer) receives the number of waits that expired
 *       on the current device since the library was loaded.
 * Both synchronise the device.
 */
int adr_decode_read_status(const void *workspace, size_t workspace_bytes, int B, int Hq, int d, int max_seq_len,
                           int partition_tokens, uint32_t *expired_waits);
int adr_stream_fault_count(uint64_t *count);

/*
 * Which kernel a pass of this shape and these flags runs on: ADR_KERNEL_VALU, ADR_KERNEL_MFMA
 * (the resident matrix-core kernel) or ADR_KERNEL_MFMA_GRID, or minus an adr_status when the
 * arguments are rejected.  The same decision adr_decode_attention takes.  adr_kernel_name gives
 * the kernel's name as profilers show it (without template arguments); "" for other values.
 */
int adr_decode_kernel_choice(const adr_kv_cache *cache, int B, int Hq, int max_seq_len, int partition_tokens,
                             unsigned flags);
const char *adr_kernel_name(int kernel);

/*
 * Debug build of the library (compiled with -DADR_DEBUG_BOUNDS; `python -m
 * paper_2503_20552_amd.build --debug` writes it next to the release library): table entries
 * and append positions that fall outside the pool or the table are counted and the first one is
 * kept.  The kernels treat them exactly as the release build does (page ids are clamped,
 * out-of-range appends are skipped).  `*record` (HOST pointer) receives the device's record;
 * reset != 0 clears it afterwards.  Synchronises.  The release build returns ADR_ERR_UNSUPPORTED.
 */
typedef struct adr_bounds_record {
    uint32_t count; /* out-of-range reads / appends seen */
    int32_t kind;   /* first one: 0 none, 1 attention read a page id outside [0, num_pages),
                       2 append position outside the row's table, 3 append page id outside the pool */
    int32_t row;    /* its request row */
    int32_t index;  /* kind 1, 3: index into the row's table; kind 2: the position */
    int32_t value;  /* kind 1, 3: the page id found; kind 2: tokens the table can describe */
} adr_bounds_record;
int adr_debug_bounds_status(adr_bounds_record *record, int reset);

const char *adr_status_string(int status);
int adr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ADR_H */
