// Host side of the C ABI: argument checks and kernel dispatch.  The attention, append, merge and
// copy entry points only enqueue kernels: they never allocate, synchronise or copy.  (The status
// readers at the end synchronise; that is what they are for.)
#include "../../include/adr.h"
#include "adr_device.h"

#include <atomic>

namespace adr {
hipError_t launch_kv_append(const AppendParams &p, bool fp8, hipStream_t stream);
hipError_t launch_decode_valu(const DecodeParams &p, int d, bool fp8, hipStream_t stream);
hipError_t launch_decode_mfma(const DecodeParams &p, int d, hipStream_t stream);
hipError_t launch_decode_stream(const DecodeParams &p, int d, bool fp8, hipStream_t stream);
hipError_t read_stream_faults(unsigned long long *count);
bool decode_stream_supports(int d, int G, int B);
bool decode_valu_supports(int d, int G);
bool decode_mfma_supports(int d, int G);
hipError_t launch_lse_merge(const MergeParams &p, hipStream_t stream);
hipError_t launch_stream_read(const void *src, size_t bytes, void *sink, hipStream_t stream);
hipError_t launch_copy(void *dst, const void *src, size_t bytes, hipStream_t stream);
} // namespace adr

namespace {

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

int check_cache(const adr_kv_cache *c)
{
    if (!c || !c->k || !c->v)
        return ADR_ERR_NULL;
    if (c->num_pages <= 0 || c->Hkv <= 0)
        return ADR_ERR_SHAPE;
    if ((c->page_size != 16 && c->page_size != 32 && c->page_size != 64) || (c->d != 64 && c->d != 128))
        return ADR_ERR_UNSUPPORTED;
    if (c->dtype != ADR_BF16 && c->dtype != ADR_FP8_E4M3)
        return ADR_ERR_UNSUPPORTED;
    if (c->dtype == ADR_FP8_E4M3 && (!c->k_scale || !c->v_scale))
        return ADR_ERR_NULL;
    if (!aligned16(c->k) || !aligned16(c->v))
        return ADR_ERR_SHAPE;
    return ADR_OK;
}

int64_t max_parts_for(int max_seq_len, int partition_tokens)
{
    if (partition_tokens <= 0)
        return 1;
    const int64_t n = ((int64_t)max_seq_len + partition_tokens - 1) / partition_tokens;
    return n < 1 ? 1 : n;
}

size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

// Layout of a split pass's workspace: partial outputs, their lse values, then the control area
// (one status block and one block per launch of the resident kernel: 512 rows each).
struct WorkspacePlan {
    size_t part_o_bytes = 0, part_lse_bytes = 0, control_bytes = 0;
    size_t total() const { return part_o_bytes + part_lse_bytes + control_bytes; }
    int control_words() const { return (int)(control_bytes / 4); }
};

WorkspacePlan plan_workspace(int B, int Hq, int d, int max_seq_len, int partition_tokens)
{
    WorkspacePlan w;
    if (partition_tokens < 0 || B <= 0 || Hq <= 0 || d <= 0 || max_seq_len <= 0)
        return w;
    if (partition_tokens > 0) {
        const size_t rows = (size_t)B * (size_t)max_parts_for(max_seq_len, partition_tokens) * Hq;
        w.part_o_bytes = round256(rows * d * sizeof(float));
        w.part_lse_bytes = round256(rows * sizeof(float));
    }
    w.control_bytes = (size_t)adr::kControlBlockBytes * (1 + (B + 511) / 512);
    return w;
}

// Clears a call's control area when no append kernel of the same call does it on its way.
__global__ void control_clear_kernel(uint32_t *words, int n)
{
    for (int i = threadIdx.x; i < n; i += blockDim.x)
        words[i] = 0u;
}

// ---- per-device addresses of this file's static device data -------------------------------
// adr_decode_attention_static keeps its workspace in `scratch`, a static device array, because
// its callers cannot allocate.  In host code the name of a static device variable is only a
// handle: the address a kernel (or a copy) may use comes from hipGetSymbolAddress, once per
// device with that device current (every device holds its own copy of the array at its own
// address).  Everything below uses those addresses, never the names.
static __device__ __align__(256) unsigned char scratch[ADR_STATIC_SCRATCH_BYTES];
#ifdef ADR_DEBUG_BOUNDS
static __device__ adr::BoundsRecord g_bounds;
#endif

struct DeviceData {
    unsigned char *scratch = nullptr;
    adr::BoundsRecord *bounds = nullptr;
};
DeviceData g_device_data[64];
std::atomic<int> g_device_ready[64];

int device_data(const DeviceData **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return ADR_ERR_LAUNCH;
    if (!g_device_ready[dev].load(std::memory_order_acquire)) {
        DeviceData dd;
        if (hipGetSymbolAddress((void **)&dd.scratch, HIP_SYMBOL(scratch)) != hipSuccess || !dd.scratch)
            return ADR_ERR_LAUNCH;
#ifdef ADR_DEBUG_BOUNDS
        if (hipGetSymbolAddress((void **)&dd.bounds, HIP_SYMBOL(g_bounds)) != hipSuccess || !dd.bounds)
            return ADR_ERR_LAUNCH;
#endif
        g_device_data[dev] = dd; // two threads racing here write the same values
        g_device_ready[dev].store(1, std::memory_order_release);
    }
    *out = &g_device_data[dev];
    return ADR_OK;
}

// Where a debug build records out-of-range table entries and positions (nullptr in a release build).
int bounds_record(adr::BoundsRecord **out)
{
    *out = nullptr;
#ifdef ADR_DEBUG_BOUNDS
    const DeviceData *dd = nullptr;
    const int rc = device_data(&dd);
    if (rc != ADR_OK)
        return rc;
    *out = dd->bounds;
#endif
    return ADR_OK;
}

} // namespace

extern "C" {

int adr_version(void) { return 200; }

int adr_stream_create_cu_mask(void **stream, const uint32_t *cu_mask, int n_words)
{
    if (!stream || !cu_mask)
        return ADR_ERR_NULL;
    if (n_words <= 0)
        return ADR_ERR_SHAPE;
    uint32_t any = 0;
    for (int i = 0; i < n_words; ++i)
        any |= cu_mask[i];
    if (!any)
        return ADR_ERR_SHAPE;
    hipStream_t s = nullptr;
    if (hipExtStreamCreateWithCUMask(&s, (uint32_t)n_words, cu_mask) != hipSuccess)
        return ADR_ERR_LAUNCH;
    *stream = (void *)s;
    return ADR_OK;
}

int adr_stream_destroy(void *stream)
{
    if (!stream)
        return ADR_ERR_NULL;
    return hipStreamDestroy((hipStream_t)stream) == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
}

int adr_stream_fault_count(uint64_t *count)
{
    if (!count)
        return ADR_ERR_NULL;
    unsigned long long n = 0;
    if (adr::read_stream_faults(&n) != hipSuccess)
        return ADR_ERR_LAUNCH;
    *count = (uint64_t)n;
    return ADR_OK;
}

const char *adr_status_string(int status)
{
    switch (status) {
    case ADR_OK: return "ok";
    case ADR_ERR_NULL: return "a required pointer is NULL";
    case ADR_ERR_SHAPE: return "a size is non-positive, inconsistent or misaligned";
    case ADR_ERR_UNSUPPORTED: return "shape or dtype outside the supported set";
    case ADR_ERR_WORKSPACE: return "workspace missing or too small for the split pass";
    case ADR_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    default: return "unknown status";
    }
}

int adr_kv_append(const adr_kv_cache *cache, const void *k_new, const void *v_new,
                  int64_t new_row_stride, const int32_t *block_table, int max_pages_per_req,
                  const int32_t *positions, int B, void *stream)
{
    const int rc = check_cache(cache);
    if (rc != ADR_OK)
        return rc;
    if (!k_new || !v_new || !block_table || !positions)
        return ADR_ERR_NULL;
    if (B < 0 || max_pages_per_req <= 0 || new_row_stride < (int64_t)cache->Hkv * cache->d)
        return ADR_ERR_SHAPE;
    if (!aligned16(k_new) || !aligned16(v_new) || (new_row_stride % 8) != 0)
        return ADR_ERR_SHAPE;
    adr::AppendParams p;
    p.k_cache = cache->k;
    p.v_cache = cache->v;
    p.k_scale = cache->k_scale;
    p.v_scale = cache->v_scale;
    p.k_new = (const uint16_t *)k_new;
    p.v_new = (const uint16_t *)v_new;
    p.new_row_stride = new_row_stride;
    p.block_table = block_table;
    p.positions = positions;
    p.seq_lens = nullptr;
    p.max_seq_len = 0;
    p.page_size = cache->page_size;
    p.max_pages = max_pages_per_req;
    p.num_pages = cache->num_pages;
    p.Hkv = cache->Hkv;
    p.d = cache->d;
    p.B = B;
    p.clear_words = nullptr;
    p.n_clear_words = 0;
    if (bounds_record(&p.bounds) != ADR_OK)
        return ADR_ERR_LAUNCH;
    const hipError_t e =
        adr::launch_kv_append(p, cache->dtype == ADR_FP8_E4M3, (hipStream_t)stream);
    return e == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
}

size_t adr_decode_workspace_bytes(int B, int Hq, int d, int max_seq_len, int partition_tokens)
{
    return plan_workspace(B, Hq, d, max_seq_len, partition_tokens).total();
}

namespace {
// The step's new token, when the call appends before it attends (adr_decode_step).
struct NewToken {
    const void *k, *v;
    int64_t row_stride;
};

// Which kernel serves a pass (negative: the status to return).
enum { KERNEL_VALU = ADR_KERNEL_VALU, KERNEL_STREAM = ADR_KERNEL_MFMA, KERNEL_GRID = ADR_KERNEL_MFMA_GRID };

int choose_kernel(const adr_kv_cache *cache, int B, int Hq, int max_seq_len, int partition_tokens, unsigned flags)
{
    const int G = Hq / cache->Hkv;
    const int d = cache->d;
    const unsigned want = flags & 0xFu;
    const bool fp8 = cache->dtype == ADR_FP8_E4M3;
    if (want == ADR_KERNEL_VALU)
        return adr::decode_valu_supports(d, G) ? KERNEL_VALU : -ADR_ERR_UNSUPPORTED;
    if (want == ADR_KERNEL_MFMA_GRID)
        return !fp8 && adr::decode_mfma_supports(d, G) ? KERNEL_GRID : -ADR_ERR_UNSUPPORTED;
    if (want == ADR_KERNEL_MFMA) {
        if (adr::decode_stream_supports(d, G, B))
            return KERNEL_STREAM;
        return !fp8 && adr::decode_mfma_supports(d, G) ? KERNEL_GRID : -ADR_ERR_UNSUPPORTED;
    }
    if (want != ADR_KERNEL_AUTO)
        return -ADR_ERR_UNSUPPORTED;
    // Measured on MI355X: the resident-workgroup kernel wins on split passes with many items
    // (groups of up to four heads always; wider groups from 2048 (request, kv-head) pairs
    // on: +11 % at 256 requests x 8 kv-heads, G = 8; about even at a quarter of that);
    // whole-row items and small passes of wide groups run faster one workgroup per item, unless
    // the bound on the lengths allows more than 32 partitions per row: that kernel's grid is sized
    // from the bound, and on the 70B-shaped workload under a bound of 32 K tokens its workgroups
    // without a partition make it 90 us against the resident kernel's 84 us (73 us under the
    // lengths' own maximum).
    const bool splits = partition_tokens > 0 && max_seq_len > partition_tokens;
    const bool many = (int64_t)B * cache->Hkv >= 2048 || max_parts_for(max_seq_len, partition_tokens) > 32;
    // An fp8 cache has the resident-workgroup kernel and the vector-ALU one only.
    if ((fp8 || (splits && (G <= 4 || many))) && adr::decode_stream_supports(d, G, B))
        return KERNEL_STREAM;
    if (!fp8 && adr::decode_mfma_supports(d, G))
        return KERNEL_GRID;
    if (adr::decode_valu_supports(d, G))
        return KERNEL_VALU;
    return -ADR_ERR_UNSUPPORTED;
}

constexpr unsigned kFlagBits = 0xFu | ADR_PARTIALS_ONLY | ADR_SINGLE_PARTITION_ITEMS | ADR_WORKSPACE_READY |
                               ADR_DEBUG_EXPIRE_WAITS | (0xFFFu << 16);

int decode_attention(void *out, adr_dtype out_dtype, float *lse, const void *q, int64_t q_row_stride,
                     const adr_kv_cache *cache, const int32_t *block_table, int max_pages_per_req,
                     const int32_t *seq_lens, int B, int Hq, float scale, int max_seq_len,
                     int partition_tokens, void *workspace, size_t workspace_bytes, unsigned flags,
                     void *stream, const NewToken *nt, bool static_scratch = false)
{
    const int rc = check_cache(cache);
    if (rc != ADR_OK)
        return rc;
    if (!out || !q || !block_table || !seq_lens)
        return ADR_ERR_NULL;
    if (nt) {
        if (!nt->k || !nt->v)
            return ADR_ERR_NULL;
        if (nt->row_stride < (int64_t)cache->Hkv * cache->d || (nt->row_stride % 8) != 0 ||
            !aligned16(nt->k) || !aligned16(nt->v))
            return ADR_ERR_SHAPE;
    }
    if (B < 0 || Hq <= 0 || max_pages_per_req <= 0 || max_seq_len < 0)
        return ADR_ERR_SHAPE;
    if (Hq % cache->Hkv != 0 || q_row_stride < (int64_t)Hq * cache->d || (q_row_stride % 8) != 0)
        return ADR_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(out))
        return ADR_ERR_SHAPE;
    if ((int64_t)max_seq_len > (int64_t)max_pages_per_req * cache->page_size)
        return ADR_ERR_SHAPE; // the table cannot describe that many tokens
    if (out_dtype != ADR_BF16 && out_dtype != ADR_F32)
        return ADR_ERR_UNSUPPORTED;
    if (partition_tokens < 0 || partition_tokens % cache->page_size != 0)
        return ADR_ERR_SHAPE;
    if (flags & ~kFlagBits)
        return ADR_ERR_UNSUPPORTED;
    const int G = Hq / cache->Hkv;
    const int d = cache->d;
    const bool fp8 = cache->dtype == ADR_FP8_E4M3;
    const int kernel = choose_kernel(cache, B, Hq, max_seq_len, partition_tokens, flags);
    if (kernel < 0)
        return -kernel;
    const int64_t max_parts = max_parts_for(max_seq_len, partition_tokens);
    if ((int64_t)B * cache->Hkv * (max_parts + 1) > 0x7fffffffLL) // (+1: the grids take an odd number per row)
        return ADR_ERR_SHAPE;
    const bool split = partition_tokens > 0 && max_parts > 1;
    const WorkspacePlan plan = plan_workspace(B, Hq, d, max_seq_len, partition_tokens);
    if (static_scratch) { // the library's own array stands in for the caller's workspace
        if (plan.total() > (size_t)ADR_STATIC_SCRATCH_BYTES)
            return ADR_ERR_WORKSPACE;
        if (flags & ADR_WORKSPACE_READY)
            return ADR_ERR_UNSUPPORTED; // calls of other sizes keep their control areas elsewhere in the array
        if (B == 0)
            return ADR_OK;
        const DeviceData *dd = nullptr;
        const int drc = device_data(&dd);
        if (drc != ADR_OK)
            return drc;
        workspace = dd->scratch;
        workspace_bytes = ADR_STATIC_SCRATCH_BYTES;
    }
    const bool workspace_fits =
        workspace && ((uintptr_t)workspace & 255u) == 0 && plan.total() > 0 && workspace_bytes >= plan.total();
    if (split && !workspace_fits)
        return ADR_ERR_WORKSPACE;
    if (B == 0)
        return ADR_OK;

    adr::DecodeParams p;
    p.q = (const uint16_t *)q;
    p.q_row_stride = q_row_stride;
    p.k_cache = cache->k;
    p.v_cache = cache->v;
    p.k_scale = cache->k_scale;
    p.v_scale = cache->v_scale;
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.out = out;
    p.lse = lse;
    p.part_o = nullptr;
    p.part_lse = nullptr;
    if (split) {
        p.part_o = (float *)workspace;
        p.part_lse = (float *)((char *)workspace + plan.part_o_bytes);
    }
    // A workspace that is large enough also carries the call's control area (an unsplit pass
    // may come with one too); a call without one falls back on the library's static pool.
    p.control = workspace_fits ? (uint32_t *)((char *)workspace + plan.part_o_bytes + plan.part_lse_bytes) : nullptr;
    p.max_pages = max_pages_per_req;
    p.page_shift = cache->page_size == 16 ? 0 : cache->page_size == 32 ? 1 : 2;
    p.B = B;
    p.Hq = Hq;
    p.Hkv = cache->Hkv;
    p.G = G;
    p.num_pages = cache->num_pages;
    p.partition_tokens = split ? partition_tokens : 0;
    p.max_parts = split ? (int)max_parts : 1;
    p.max_seq_len = max_seq_len;
    p.out_f32 = out_dtype == ADR_F32;
    p.scale_log2e = scale * adr::kLog2e;
    p.coalesce = !(flags & ADR_SINGLE_PARTITION_ITEMS);
    p.spin_limit = (flags & ADR_DEBUG_EXPIRE_WAITS) ? 0 : adr::kSpinLimit;
    p.grid_cus = (int)((flags >> 16) & 0xFFFu);
    if (bounds_record(&p.bounds) != ADR_OK)
        return ADR_ERR_LAUNCH;

    // The control area must be all zero when the resident kernel starts and when a merge reads the
    // status block.  Kernels that never touch it leave the merge without a status to read.
    const bool uses_control = p.control && (kernel == KERNEL_STREAM || (flags & ADR_PARTIALS_ONLY));
    const bool clear_control = uses_control && !(flags & ADR_WORKSPACE_READY);

    // The new token goes in first: the append kernel, with the token index taken from seq_lens.
    if (nt) {
        adr::AppendParams ap;
        ap.k_cache = cache->k;
        ap.v_cache = cache->v;
        ap.k_scale = cache->k_scale;
        ap.v_scale = cache->v_scale;
        ap.k_new = (const uint16_t *)nt->k;
        ap.v_new = (const uint16_t *)nt->v;
        ap.new_row_stride = nt->row_stride;
        ap.block_table = block_table;
        ap.positions = nullptr;
        ap.seq_lens = seq_lens;
        ap.max_seq_len = max_seq_len;
        ap.page_size = cache->page_size;
        ap.max_pages = max_pages_per_req;
        ap.num_pages = cache->num_pages;
        ap.Hkv = cache->Hkv;
        ap.d = d;
        ap.B = B;
        ap.clear_words = clear_control ? p.control : nullptr; // on its way, for the kernels behind it
        ap.n_clear_words = clear_control ? plan.control_words() : 0;
        ap.bounds = p.bounds;
        if (adr::launch_kv_append(ap, fp8, (hipStream_t)stream) != hipSuccess)
            return ADR_ERR_LAUNCH;
    } else if (clear_control) {
        control_clear_kernel<<<1, 64, 0, (hipStream_t)stream>>>(p.control, plan.control_words());
        if (hipGetLastError() != hipSuccess)
            return ADR_ERR_LAUNCH;
    }
    hipError_t e = kernel == KERNEL_STREAM ? adr::launch_decode_stream(p, d, fp8, (hipStream_t)stream)
                   : kernel == KERNEL_GRID ? adr::launch_decode_mfma(p, d, (hipStream_t)stream)
                                           : adr::launch_decode_valu(p, d, fp8, (hipStream_t)stream);
    if (e != hipSuccess)
        return ADR_ERR_LAUNCH;
    if (split && !(flags & ADR_PARTIALS_ONLY)) {
        adr::MergeParams mp;
        mp.out = out;
        mp.lse_out = lse;
        mp.part_o = p.part_o;
        mp.part_lse = p.part_lse;
        mp.part_offsets = nullptr;
        mp.seq_lens = seq_lens;
        mp.partition_tokens = partition_tokens;
        mp.max_parts = (int)max_parts;
        mp.max_seq_len = max_seq_len;
        mp.B = B;
        mp.heads = Hq;
        mp.d = d;
        mp.out_f32 = p.out_f32;
        mp.status = uses_control ? p.control : nullptr;
        e = adr::launch_lse_merge(mp, (hipStream_t)stream);
        if (e != hipSuccess)
            return ADR_ERR_LAUNCH;
    }
    return ADR_OK;
}

} // namespace

int adr_decode_attention(void *out, adr_dtype out_dtype, float *lse, const void *q,
                         int64_t q_row_stride, const adr_kv_cache *cache,
                         const int32_t *block_table, int max_pages_per_req,
                         const int32_t *seq_lens, int B, int Hq, float scale, int max_seq_len,
                         int partition_tokens, void *workspace, size_t workspace_bytes,
                         unsigned flags, void *stream)
{
    return decode_attention(out, out_dtype, lse, q, q_row_stride, cache, block_table, max_pages_per_req,
                            seq_lens, B, Hq, scale, max_seq_len, partition_tokens, workspace,
                            workspace_bytes, flags, stream, nullptr);
}

int adr_decode_attention_static(void *out, adr_dtype out_dtype, float *lse, const void *q, int64_t q_row_stride,
                                const adr_kv_cache *cache, const int32_t *block_table, int max_pages_per_req,
                                const int32_t *seq_lens, int B, int Hq, float scale, int max_seq_len,
                                int partition_tokens, unsigned flags, void *stream)
{
    return decode_attention(out, out_dtype, lse, q, q_row_stride, cache, block_table, max_pages_per_req,
                            seq_lens, B, Hq, scale, max_seq_len, partition_tokens, nullptr, 0, flags, stream,
                            nullptr, true);
}

int adr_decode_step(void *out, adr_dtype out_dtype, float *lse, const void *q, int64_t q_row_stride,
                    const void *k_new, const void *v_new, int64_t new_row_stride,
                    const adr_kv_cache *cache, const int32_t *block_table, int max_pages_per_req,
                    const int32_t *seq_lens, int B, int Hq, float scale, int max_seq_len,
                    int partition_tokens, void *workspace, size_t workspace_bytes, unsigned flags,
                    void *stream)
{
    const NewToken nt = {k_new, v_new, new_row_stride};
    return decode_attention(out, out_dtype, lse, q, q_row_stride, cache, block_table, max_pages_per_req,
                            seq_lens, B, Hq, scale, max_seq_len, partition_tokens, workspace,
                            workspace_bytes, flags, stream, &nt);
}

int adr_decode_merge(void *out, adr_dtype out_dtype, float *lse, const int32_t *seq_lens, int B,
                     int Hq, int d, int max_seq_len, int partition_tokens, const void *workspace,
                     size_t workspace_bytes, void *stream)
{
    if (!out || !seq_lens)
        return ADR_ERR_NULL;
    if (B < 0 || Hq <= 0 || max_seq_len < 0 || partition_tokens < 0 ||
        partition_tokens % adr::kPageSize != 0 || !aligned16(out))
        return ADR_ERR_SHAPE;
    if (d != 64 && d != 128)
        return ADR_ERR_UNSUPPORTED;
    if (out_dtype != ADR_BF16 && out_dtype != ADR_F32)
        return ADR_ERR_UNSUPPORTED;
    const int64_t max_parts = max_parts_for(max_seq_len, partition_tokens);
    if (partition_tokens == 0 || max_parts <= 1 || B == 0)
        return ADR_OK;
    const WorkspacePlan plan = plan_workspace(B, Hq, d, max_seq_len, partition_tokens);
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < plan.total())
        return ADR_ERR_WORKSPACE;
    adr::MergeParams mp;
    mp.out = out;
    mp.lse_out = lse;
    mp.part_o = (const float *)workspace;
    mp.part_lse = (const float *)((const char *)workspace + plan.part_o_bytes);
    mp.status = (const uint32_t *)((const char *)workspace + plan.part_o_bytes + plan.part_lse_bytes);
    mp.part_offsets = nullptr;
    mp.seq_lens = seq_lens;
    mp.partition_tokens = partition_tokens;
    mp.max_parts = (int)max_parts;
    mp.max_seq_len = max_seq_len;
    mp.B = B;
    mp.heads = Hq;
    mp.d = d;
    mp.out_f32 = out_dtype == ADR_F32;
    return adr::launch_lse_merge(mp, (hipStream_t)stream) == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
}

int adr_lse_merge(void *out, adr_dtype out_dtype, float *lse_out, const float *part_o,
                  const float *part_lse, const int32_t *part_offsets, int B, int heads, int d,
                  void *stream)
{
    if (!out || !part_o || !part_lse || !part_offsets)
        return ADR_ERR_NULL;
    if (B < 0 || heads <= 0)
        return ADR_ERR_SHAPE;
    if (d != 64 && d != 128)
        return ADR_ERR_UNSUPPORTED;
    if (out_dtype != ADR_BF16 && out_dtype != ADR_F32)
        return ADR_ERR_UNSUPPORTED;
    if (!aligned16(out) || !aligned16(part_o))
        return ADR_ERR_SHAPE;
    adr::MergeParams mp;
    mp.out = out;
    mp.lse_out = lse_out;
    mp.part_o = part_o;
    mp.part_lse = part_lse;
    mp.part_offsets = part_offsets;
    mp.seq_lens = nullptr;
    mp.partition_tokens = 0;
    mp.max_parts = 0;
    mp.max_seq_len = 0;
    mp.B = B;
    mp.heads = heads;
    mp.d = d;
    mp.out_f32 = out_dtype == ADR_F32;
    mp.status = nullptr;
    return adr::launch_lse_merge(mp, (hipStream_t)stream) == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
}

int adr_decode_kernel_choice(const adr_kv_cache *cache, int B, int Hq, int max_seq_len, int partition_tokens,
                             unsigned flags)
{
    const int rc = check_cache(cache);
    if (rc != ADR_OK)
        return -rc;
    if (B < 0 || Hq <= 0 || Hq % cache->Hkv != 0 || max_seq_len < 0 || partition_tokens < 0)
        return -ADR_ERR_SHAPE;
    return choose_kernel(cache, B, Hq, max_seq_len, partition_tokens, flags);
}

const char *adr_kernel_name(int kernel)
{
    switch (kernel) {
    case ADR_KERNEL_VALU: return "decode_valu_kernel";
    case ADR_KERNEL_MFMA: return "decode_stream_kernel";
    case ADR_KERNEL_MFMA_GRID: return "decode_mfma_kernel";
    default: return "";
    }
}

int adr_decode_read_status(const void *workspace, size_t workspace_bytes, int B, int Hq, int d, int max_seq_len,
                           int partition_tokens, uint32_t *expired_waits)
{
    if (!workspace || !expired_waits)
        return ADR_ERR_NULL;
    const WorkspacePlan plan = plan_workspace(B, Hq, d, max_seq_len, partition_tokens);
    if (plan.total() == 0 || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < plan.total())
        return ADR_ERR_WORKSPACE;
    const char *status = (const char *)workspace + plan.part_o_bytes + plan.part_lse_bytes;
    uint32_t word = 0;
    if (hipMemcpy(&word, status + 4 * adr::kStatusExpiredWaits, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess)
        return ADR_ERR_LAUNCH;
    *expired_waits = word;
    return ADR_OK;
}

int adr_debug_bounds_status(adr_bounds_record *record, int reset)
{
#ifdef ADR_DEBUG_BOUNDS
    if (!record)
        return ADR_ERR_NULL;
    adr::BoundsRecord *dev = nullptr;
    if (bounds_record(&dev) != ADR_OK || !dev)
        return ADR_ERR_LAUNCH;
    adr::BoundsRecord host;
    if (hipMemcpy(&host, dev, sizeof(host), hipMemcpyDeviceToHost) != hipSuccess)
        return ADR_ERR_LAUNCH;
    record->count = host.count;
    record->kind = host.kind;
    record->row = host.row;
    record->index = host.index;
    record->value = host.value;
    if (reset && hipMemset(dev, 0, sizeof(host)) != hipSuccess)
        return ADR_ERR_LAUNCH;
    return ADR_OK;
#else
    (void)record;
    (void)reset;
    return ADR_ERR_UNSUPPORTED;
#endif
}

int adr_probe_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink)
        return ADR_ERR_NULL;
    if (bytes % 16 != 0 || !aligned16(src))
        return ADR_ERR_SHAPE;
    return adr::launch_stream_read(src, bytes, sink, (hipStream_t)stream) == hipSuccess
               ? ADR_OK
               : ADR_ERR_LAUNCH;
}

int adr_probe_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!src || !dst)
        return ADR_ERR_NULL;
    if (bytes % 16 != 0 || !aligned16(src) || !aligned16(dst))
        return ADR_ERR_SHAPE;
    return adr::launch_copy(dst, src, bytes, (hipStream_t)stream) == hipSuccess ? ADR_OK
                                                                                : ADR_ERR_LAUNCH;
}

} // extern "C"
