// Host side of the C ABI: argument checks and kernel dispatch.  Nothing here
// allocates, synchronises or copies; every entry point only enqueues kernels.
#include "../../include/adr.h"
#include "adr_device.h"

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

} // namespace

extern "C" {

int adr_version(void) { return 100; }

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
    const hipError_t e =
        adr::launch_kv_append(p, cache->dtype == ADR_FP8_E4M3, (hipStream_t)stream);
    return e == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
}

size_t adr_decode_workspace_bytes(int B, int Hq, int d, int max_seq_len, int partition_tokens)
{
    if (partition_tokens <= 0 || B <= 0 || Hq <= 0 || d <= 0 || max_seq_len <= 0)
        return 0;
    const size_t rows = (size_t)B * (size_t)max_parts_for(max_seq_len, partition_tokens) * Hq;
    return round256(rows * d * sizeof(float)) + round256(rows * sizeof(float));
}

namespace {
// The step's new token, when the call appends before it attends (adr_decode_step).
struct NewToken {
    const void *k, *v;
    int64_t row_stride;
};

int decode_attention(void *out, adr_dtype out_dtype, float *lse, const void *q, int64_t q_row_stride,
                     const adr_kv_cache *cache, const int32_t *block_table, int max_pages_per_req,
                     const int32_t *seq_lens, int B, int Hq, float scale, int max_seq_len,
                     int partition_tokens, void *workspace, size_t workspace_bytes, unsigned flags,
                     void *stream, const NewToken *nt)
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
    if (flags & ~(0xFu | ADR_PARTIALS_ONLY | ADR_SINGLE_PARTITION_ITEMS))
        return ADR_ERR_UNSUPPORTED;
    const int G = Hq / cache->Hkv;
    const int d = cache->d;
    const unsigned want = flags & 0xFu;
    const bool fp8 = cache->dtype == ADR_FP8_E4M3;
    enum { VALU, MFMA_GRID, MFMA_STREAM } kernel;
    if (want == ADR_KERNEL_VALU) {
        if (!adr::decode_valu_supports(d, G))
            return ADR_ERR_UNSUPPORTED;
        kernel = VALU;
    } else if (want == ADR_KERNEL_MFMA_GRID) {
        if (fp8 || !adr::decode_mfma_supports(d, G))
            return ADR_ERR_UNSUPPORTED;
        kernel = MFMA_GRID;
    } else if (want == ADR_KERNEL_MFMA) {
        if (adr::decode_stream_supports(d, G, B))
            kernel = MFMA_STREAM;
        else if (!fp8 && adr::decode_mfma_supports(d, G))
            kernel = MFMA_GRID;
        else
            return ADR_ERR_UNSUPPORTED;
    } else if (want == ADR_KERNEL_AUTO) {
        // Measured on MI355X: the resident-workgroup kernel wins on split passes with many items
        // (groups of up to four heads always; wider groups from 2048 (request, kv-head) pairs
        // on: +11 % at 256 requests x 8 kv-heads, G = 8; about even at a quarter of that);
        // whole-row items and small passes of wide groups run faster one workgroup per item.
        const bool splits = partition_tokens > 0 && max_seq_len > partition_tokens;
        const bool many = (int64_t)B * cache->Hkv >= 2048;
        // An fp8 cache has the resident-workgroup kernel and the vector-ALU one only.
        if ((fp8 || (splits && (G <= 4 || many))) && adr::decode_stream_supports(d, G, B))
            kernel = MFMA_STREAM;
        else if (!fp8 && adr::decode_mfma_supports(d, G))
            kernel = MFMA_GRID;
        else if (adr::decode_valu_supports(d, G))
            kernel = VALU;
        else
            return ADR_ERR_UNSUPPORTED;
    } else {
        return ADR_ERR_UNSUPPORTED;
    }
    const int64_t max_parts = max_parts_for(max_seq_len, partition_tokens);
    if ((int64_t)B * cache->Hkv * max_parts > 0x7fffffffLL)
        return ADR_ERR_SHAPE;
    const bool split = partition_tokens > 0 && max_parts > 1;
    if (split) {
        if (!workspace)
            return ADR_ERR_WORKSPACE;
        if (((uintptr_t)workspace & 255u) != 0 ||
            workspace_bytes < adr_decode_workspace_bytes(B, Hq, d, max_seq_len, partition_tokens))
            return ADR_ERR_WORKSPACE;
    }
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
        const size_t rows = (size_t)B * (size_t)max_parts * Hq;
        p.part_o = (float *)workspace;
        p.part_lse = (float *)((char *)workspace + round256(rows * d * sizeof(float)));
    }
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
        if (adr::launch_kv_append(ap, fp8, (hipStream_t)stream) != hipSuccess)
            return ADR_ERR_LAUNCH;
    }
    hipError_t e = kernel == MFMA_STREAM ? adr::launch_decode_stream(p, d, fp8, (hipStream_t)stream)
                   : kernel == MFMA_GRID ? adr::launch_decode_mfma(p, d, (hipStream_t)stream)
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
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 ||
        workspace_bytes < adr_decode_workspace_bytes(B, Hq, d, max_seq_len, partition_tokens))
        return ADR_ERR_WORKSPACE;
    const size_t rows = (size_t)B * (size_t)max_parts * Hq;
    adr::MergeParams mp;
    mp.out = out;
    mp.lse_out = lse;
    mp.part_o = (const float *)workspace;
    mp.part_lse = (const float *)((const char *)workspace + round256(rows * d * sizeof(float)));
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
    return adr::launch_lse_merge(mp, (hipStream_t)stream) == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
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
