// C ABI of the library (see include/lserve.h): host-side argument validation, translation of the
// public structs into kernel parameter blocks, and launches on the caller's stream.  No device
// memory is allocated or freed here and no state survives a call.
#include "../../include/lserve.h"

#include <cmath>
#include <mutex>

#include "kernels.h"

using namespace lserve;

// Scratch of lserve_sparse_decode_noalloc: the partial results the decode kernels exchange, which the other
// decode entry point keeps in the caller's workspace.  One copy per GPU for the life of the process.  In host code
// the name is only a handle: the address on a device comes from hipGetSymbolAddress (scratch_on_current_device).
constexpr size_t kScratchBytes = LSERVE_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

thread_local int g_last_hip_error = 0;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch`, per device, once resolved

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int fail_hip(hipError_t e) {
    g_last_hip_error = (int)e;
    return LSERVE_ERR_HIP;
}

// Address of `scratch` on the device that is current on the calling thread; resolved once per device.
int scratch_on_current_device(void** ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e);
    if (dev < 0 || dev >= kMaxDevices) return LSERVE_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return fail_hip(e);
        if (!p) return fail_hip(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return LSERVE_OK;
}

// Validates the layer description and fills the kernel parameter block.
int make_layer(const lserve_attn_desc* d, LayerParams* lp) {
    if (!d || !d->kv_head_is_streaming) return LSERVE_ERR_INVALID_ARG;
    if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->page_size <= 0 || d->logical_page_size <= 0)
        return LSERVE_ERR_INVALID_ARG;
    if (d->sink_tokens < 0 || d->local_tokens < 1) return LSERVE_ERR_INVALID_ARG;
    if (d->page_size % d->logical_page_size != 0) return LSERVE_ERR_INVALID_ARG;
    if (!(d->sm_scale >= 0.f) || std::isinf(d->sm_scale)) return LSERVE_ERR_INVALID_ARG;
    if (d->head_dim != kHeadDim) return LSERVE_ERR_UNSUPPORTED;
    if (d->dtype != LSERVE_DTYPE_FP16 && d->dtype != LSERVE_DTYPE_BF16) return LSERVE_ERR_UNSUPPORTED;
    if (d->num_q_heads % d->num_kv_heads != 0) return LSERVE_ERR_UNSUPPORTED;
    if (d->num_kv_heads > 64 || d->num_q_heads / d->num_kv_heads > kMaxGroup) return LSERVE_ERR_UNSUPPORTED;
    if (d->page_size != 16 && d->page_size != 32 && d->page_size != 64 && d->page_size != 128)
        return LSERVE_ERR_UNSUPPORTED;
    if (d->page_size / d->logical_page_size > kMaxLogical) return LSERVE_ERR_UNSUPPORTED;
    lp->H = d->num_q_heads;
    lp->Hkv = d->num_kv_heads;
    lp->group = lp->H / lp->Hkv;
    lp->NP = d->page_size;
    lp->NL = d->logical_page_size;
    lp->g = lp->NP / lp->NL;
    lp->sink_pages = (d->sink_tokens + lp->NP - 1) / lp->NP;
    lp->local_pages = (d->local_tokens + lp->NP - 1) / lp->NP;
    lp->streaming_mask = 0;
    for (int h = 0; h < lp->Hkv; ++h)
        if (d->kv_head_is_streaming[h]) lp->streaming_mask |= 1ull << h;
    const float scale = d->sm_scale > 0.f ? d->sm_scale : 1.0f / std::sqrt((float)kHeadDim);
    lp->sm_scale_log2 = scale * 1.4426950408889634f;
    return LSERVE_OK;
}

// need_stream: the call touches streaming heads, so every one of them must live in some pool.
int make_paged(const lserve_paged_kv* kv, const LayerParams& lp, bool need_k, bool need_v, bool need_stats,
               bool need_stream, PagedParams* pp) {
    if (!kv || !kv->page_table || !kv->seq_lens) return LSERVE_ERR_INVALID_ARG;
    if (kv->batch <= 0 || kv->max_pages_per_seq <= 0 || kv->num_pages <= 0) return LSERVE_ERR_INVALID_ARG;
    if (kv->batch > 65535) return LSERVE_ERR_UNSUPPORTED;
    if ((need_k && !kv->k_pool) || (need_v && !kv->v_pool) || (need_stats && !kv->stats)) return LSERVE_ERR_INVALID_ARG;
    if (!aligned16(kv->k_pool) || !aligned16(kv->v_pool) || !aligned16(kv->stats) || !aligned16(kv->page_table) ||
        !aligned16(kv->seq_lens))
        return LSERVE_ERR_INVALID_ARG;
    pp->k_pool = kv->k_pool;
    pp->v_pool = kv->v_pool;
    pp->stats = kv->stats;
    pp->page_table = kv->page_table;
    pp->seq_lens = kv->seq_lens;
    pp->batch = kv->batch;
    pp->max_pages = kv->max_pages_per_seq;
    pp->num_pages = kv->num_pages;
    int n_stream = 0;
    for (int h = 0; h < lp.Hkv; ++h) n_stream += (int)((lp.streaming_mask >> h) & 1ull);
    const int n_dense = lp.Hkv - n_stream;
    pp->pool_heads = kv->pool_heads == 0 ? lp.Hkv : kv->pool_heads;
    if (pp->pool_heads != lp.Hkv && pp->pool_heads != n_dense) return LSERVE_ERR_INVALID_ARG;
    if ((kv->k_pool_stream == nullptr) != (kv->v_pool_stream == nullptr)) return LSERVE_ERR_INVALID_ARG;
    pp->k_stream = kv->k_pool_stream;
    pp->v_stream = kv->v_pool_stream;
    pp->ring_table = kv->ring_table;
    pp->stream_heads = n_stream;
    pp->ring = lp.sink_pages + lp.local_pages;
    if (pp->k_stream) {
        if (!kv->ring_table || kv->num_pages_stream <= 0 || n_stream == 0) return LSERVE_ERR_INVALID_ARG;
        if (!aligned16(kv->k_pool_stream) || !aligned16(kv->v_pool_stream) || !aligned16(kv->ring_table))
            return LSERVE_ERR_INVALID_ARG;
    }
    if (kv->kv_bits != 0 && kv->kv_bits != 16 && kv->kv_bits != 8 && kv->kv_bits != 4) return LSERVE_ERR_INVALID_ARG;
    pp->kv_bits = kv->kv_bits == 0 ? 16 : kv->kv_bits;
    if (pp->kv_bits != 16 && lp.NP != 64) return LSERVE_ERR_UNSUPPORTED;
    const bool main_holds_all = pp->pool_heads == lp.Hkv;
    if (need_stream && n_stream > 0 && !main_holds_all && !pp->k_stream) return LSERVE_ERR_INVALID_ARG;
    return LSERVE_OK;
}

HeadList selecting_heads(const LayerParams& lp) {
    HeadList hl;
    hl.count = 0;
    for (int h = 0; h < lp.Hkv; ++h)
        if (!((lp.streaming_mask >> h) & 1ull)) hl.idx[hl.count++] = (unsigned char)h;
    return hl;
}

size_t select_workspace_bytes(const LayerParams& lp, int batch, int max_pages) {
    return (size_t)batch * lp.Hkv * max_pages * sizeof(float);
}

}  // namespace

extern "C" {

int lserve_build_page_stats(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const int32_t* start_pos,
                            int32_t max_tail_pages, void* stream) {
    LayerParams lp;
    PagedParams pp;
    int rc = make_layer(desc, &lp);
    if (rc) return rc;
    rc = make_paged(kv, lp, true, false, true, false, &pp);
    if (rc) return rc;
    if (pp.kv_bits != 16) return LSERVE_ERR_UNSUPPORTED;  // statistics come from 16-bit keys (lserve_append_kv)
    if (max_tail_pages < 0 || !aligned16(start_pos)) return LSERVE_ERR_INVALID_ARG;
    const int tail = (max_tail_pages == 0 || max_tail_pages > pp.max_pages) ? pp.max_pages : max_tail_pages;
    hipError_t e = launch_page_stats(desc->dtype, lp, pp, start_pos, tail, selecting_heads(lp), (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

int lserve_append_kv(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const void* k_new, const void* v_new,
                     const int32_t* cu_new, const int32_t* start_pos, int32_t max_new_per_seq, void* stream) {
    LayerParams lp;
    PagedParams pp;
    int rc = make_layer(desc, &lp);
    if (rc) return rc;
    rc = make_paged(kv, lp, true, true, selecting_heads(lp).count > 0, true, &pp);
    if (rc) return rc;
    if (!k_new || !v_new || !cu_new || !start_pos || max_new_per_seq <= 0) return LSERVE_ERR_INVALID_ARG;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(cu_new) || !aligned16(start_pos)) return LSERVE_ERR_INVALID_ARG;
    hipError_t e = launch_append_kv(desc->dtype, lp, pp, k_new, v_new, cu_new, start_pos, max_new_per_seq,
                                    (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

int lserve_select_pages(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const void* q, int32_t budget_tokens,
                        const int32_t* stats_valid_len, int32_t* sel_pages, int32_t* sel_count, int32_t* sel_seq_len,
                        float* scores_out, void* workspace, size_t workspace_bytes, void* stream) {
    LayerParams lp;
    PagedParams pp;
    int rc = make_layer(desc, &lp);
    if (rc) return rc;
    rc = make_paged(kv, lp, stats_valid_len != nullptr, false, selecting_heads(lp).count > 0, false, &pp);
    if (rc) return rc;
    if (stats_valid_len && pp.kv_bits != 16) return LSERVE_ERR_UNSUPPORTED;  // no 16-bit keys to rebuild from
    if (!q || !sel_pages || !sel_count || !sel_seq_len) return LSERVE_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(stats_valid_len) || !aligned16(sel_pages) || !aligned16(sel_count) || !aligned16(sel_seq_len) ||
        !aligned16(scores_out) || !aligned16(workspace))
        return LSERVE_ERR_INVALID_ARG;
    if (budget_tokens < lp.NP) return LSERVE_ERR_INVALID_ARG;
    float* scores = scores_out;
    if (!scores) {
        if (!workspace || workspace_bytes < select_workspace_bytes(lp, pp.batch, pp.max_pages)) return LSERVE_ERR_WORKSPACE;
        scores = reinterpret_cast<float*>(workspace);
    }
    hipError_t e = launch_select_pages(desc->dtype, lp, pp, q, stats_valid_len, budget_tokens / lp.NP, sel_pages, sel_count,
                                       sel_seq_len, scores, scores_out != nullptr, selecting_heads(lp), (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

namespace {
int prefill_impl(const lserve_attn_desc* desc, const lserve_block_mask* mask, const void* q, const void* k, const void* v,
                 const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen, void* out,
                 float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
    LayerParams lp;
    int rc = make_layer(desc, &lp);
    if (rc) return rc;
    if (!q || !k || !v || !cu_seqlens || !out) return LSERVE_ERR_INVALID_ARG;
    if (batch <= 0 || total_tokens <= 0 || max_seqlen <= 0 || max_seqlen > total_tokens) return LSERVE_ERR_INVALID_ARG;
    if (batch > 65535) return LSERVE_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(cu_seqlens) ||
        !aligned16(lse_out) || !aligned16(workspace))
        return LSERVE_ERR_INVALID_ARG;
    if (lp.NP != 64) return LSERVE_ERR_UNSUPPORTED;
    PrefillMaskArgs ma = {};
    size_t need = prefill_workspace_bytes(lp, total_tokens, batch);
    if (mask) {
        if (!mask->head_mask || !mask->q_tile_start || !mask->row_ptr || (mask->nnz > 0 && !mask->cols))
            return LSERVE_ERR_INVALID_ARG;
        if (mask->num_masks <= 0 || mask->rows_per_mask <= 0 || mask->nnz < 0) return LSERVE_ERR_INVALID_ARG;
        if (!aligned16(mask->head_mask) || !aligned16(mask->q_tile_start) || !aligned16(mask->row_ptr) ||
            !aligned16(mask->cols))
            return LSERVE_ERR_INVALID_ARG;
        if (max_seqlen > 65536 * 64) return LSERVE_ERR_UNSUPPORTED;  // one byte of LDS per key tile in the merge pass
        ma.head_mask = mask->head_mask;
        ma.q_tile_start = mask->q_tile_start;
        ma.row_ptr = mask->row_ptr;
        ma.cols = mask->cols;
        ma.num_masks = mask->num_masks;
        ma.rows_per_mask = mask->rows_per_mask;
        ma.nnz = mask->nnz;
        need = masked_prefill_workspace_bytes(lp, total_tokens, batch, max_seqlen, mask->num_masks, mask->nnz);
    }
    if (need > 0 && (!workspace || workspace_bytes < need)) return LSERVE_ERR_WORKSPACE;
    hipError_t e = launch_sparse_prefill(desc->dtype, lp, q, k, v, cu_seqlens, batch, total_tokens, max_seqlen, out,
                                         lse_out, workspace, mask ? &ma : nullptr, (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}
}  // namespace

int lserve_sparse_prefill(const lserve_attn_desc* desc, const void* q, const void* k, const void* v,
                          const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen, void* out,
                          float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
    return prefill_impl(desc, nullptr, q, k, v, cu_seqlens, batch, total_tokens, max_seqlen, out, lse_out, workspace,
                        workspace_bytes, stream);
}

int lserve_sparse_prefill_masked(const lserve_attn_desc* desc, const lserve_block_mask* mask, const void* q, const void* k,
                                 const void* v, const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens,
                                 int32_t max_seqlen, void* out, float* lse_out, void* workspace, size_t workspace_bytes,
                                 void* stream) {
    if (!mask) return LSERVE_ERR_INVALID_ARG;
    return prefill_impl(desc, mask, q, k, v, cu_seqlens, batch, total_tokens, max_seqlen, out, lse_out, workspace,
                        workspace_bytes, stream);
}

int lserve_sparse_prefill_paged(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const void* q,
                                const int32_t* cu_q, int32_t total_new, int32_t max_new_per_seq, int32_t max_seqlen,
                                void* out, float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
    LayerParams lp;
    PagedParams pp;
    int rc = make_layer(desc, &lp);
    if (rc) return rc;
    rc = make_paged(kv, lp, true, true, false, true, &pp);
    if (rc) return rc;
    if (lp.NP != 64) return LSERVE_ERR_UNSUPPORTED;
    if (pp.pool_heads != lp.Hkv || pp.k_stream) return LSERVE_ERR_UNSUPPORTED;  // one pool holding every head
    if (pp.kv_bits != 16) return LSERVE_ERR_UNSUPPORTED;
    if (!q || !cu_q || !out) return LSERVE_ERR_INVALID_ARG;
    if (total_new <= 0 || max_new_per_seq <= 0 || max_new_per_seq > total_new || max_seqlen < max_new_per_seq)
        return LSERVE_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(cu_q) || !aligned16(out) || !aligned16(lse_out) || !aligned16(workspace))
        return LSERVE_ERR_INVALID_ARG;
    const size_t need = paged_prefill_workspace_bytes(lp, pp.batch, pp.max_pages);
    if (need > 0 && (!workspace || workspace_bytes < need)) return LSERVE_ERR_WORKSPACE;
    hipError_t e = launch_sparse_prefill_paged(desc->dtype, lp, pp, q, nullptr, nullptr, cu_q, total_new, max_new_per_seq,
                                               max_seqlen, out, lse_out, workspace, (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

int lserve_sparse_prefill_chunk(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const void* q, const void* k_new,
                                const void* v_new, const int32_t* cu_new, int32_t total_new, int32_t max_new_per_seq,
                                void* out, float* lse_out, void* stream) {
    LayerParams lp;
    PagedParams pp;
    int rc = make_layer(desc, &lp);
    if (rc) return rc;
    rc = make_paged(kv, lp, true, true, false, true, &pp);
    if (rc) return rc;
    if (lp.NP != 64) return LSERVE_ERR_UNSUPPORTED;
    if (!q || !k_new || !v_new || !cu_new || !out) return LSERVE_ERR_INVALID_ARG;
    if (total_new <= 0 || max_new_per_seq <= 0 || max_new_per_seq > total_new) return LSERVE_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(cu_new) || !aligned16(out) ||
        !aligned16(lse_out))
        return LSERVE_ERR_INVALID_ARG;
    hipError_t e = launch_sparse_prefill_paged(desc->dtype, lp, pp, q, k_new, v_new, cu_new, total_new, max_new_per_seq, 0,
                                               out, lse_out, nullptr, (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

size_t lserve_paged_prefill_workspace_bytes(const lserve_attn_desc* desc, int32_t batch, int32_t max_pages_per_seq) {
    LayerParams lp;
    if (make_layer(desc, &lp) != LSERVE_OK || batch <= 0 || max_pages_per_seq <= 0) return 0;
    return paged_prefill_workspace_bytes(lp, batch, max_pages_per_seq);
}

size_t lserve_masked_prefill_workspace_bytes(const lserve_attn_desc* desc, int32_t batch, int32_t total_tokens,
                                             int32_t max_seqlen, int32_t num_masks, int32_t nnz) {
    LayerParams lp;
    if (make_layer(desc, &lp) != LSERVE_OK) return 0;
    if (batch <= 0 || total_tokens <= 0 || max_seqlen <= 0 || num_masks <= 0 || nnz < 0) return 0;
    return masked_prefill_workspace_bytes(lp, total_tokens, batch, max_seqlen, num_masks, nnz);
}

namespace {
// Everything lserve_sparse_decode checks except the workspace.
int check_decode_args(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const void* q, const int32_t* sel_pages,
                      const int32_t* sel_count, const int32_t* sel_seq_len, int32_t sel_stride, const void* out,
                      const float* lse_out, LayerParams* lp, PagedParams* pp) {
    int rc = make_layer(desc, lp);
    if (rc) return rc;
    rc = make_paged(kv, *lp, true, true, false, true, pp);
    if (rc) return rc;
    if (!q || !out) return LSERVE_ERR_INVALID_ARG;
    const bool any_selecting = selecting_heads(*lp).count > 0;
    if (any_selecting && (!sel_pages || !sel_count || !sel_seq_len || sel_stride <= 0)) return LSERVE_ERR_INVALID_ARG;
    if (sel_stride < 0) return LSERVE_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(out) || !aligned16(sel_pages) || !aligned16(sel_count) || !aligned16(sel_seq_len) ||
        !aligned16(lse_out))
        return LSERVE_ERR_INVALID_ARG;
    // the launch plan numbers the nominal index-table entries of the whole batch with 32-bit integers
    if ((long long)pp->batch * decode_nominal_entries(*lp, sel_stride) > 0x7fffffffLL) return LSERVE_ERR_UNSUPPORTED;
    return LSERVE_OK;
}
}  // namespace

int lserve_sparse_decode(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const void* q,
                         const int32_t* sel_pages, const int32_t* sel_count, const int32_t* sel_seq_len,
                         int32_t sel_stride, void* out, float* lse_out, void* workspace, size_t workspace_bytes,
                         void* stream) {
    LayerParams lp;
    PagedParams pp;
    int rc = check_decode_args(desc, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out, lse_out, &lp, &pp);
    if (rc) return rc;
    if (!aligned16(workspace)) return LSERVE_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < decode_workspace_bytes(lp, pp.batch, sel_stride)) return LSERVE_ERR_WORKSPACE;
    hipError_t e = launch_sparse_decode(desc->dtype, lp, pp, q, sel_pages, sel_count, sel_seq_len, sel_stride, out,
                                        lse_out, workspace, (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

int lserve_sparse_decode_noalloc(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const void* q,
                                 const int32_t* sel_pages, const int32_t* sel_count, const int32_t* sel_seq_len,
                                 int32_t sel_stride, void* out, float* lse_out, void* stream) {
    LayerParams lp;
    PagedParams pp;
    int rc = check_decode_args(desc, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out, lse_out, &lp, &pp);
    if (rc) return rc;
    if (decode_workspace_bytes(lp, pp.batch, sel_stride) > kScratchBytes) return LSERVE_ERR_WORKSPACE;
    void* ws = nullptr;
    rc = scratch_on_current_device(&ws);
    if (rc) return rc;
    // The arrival counters at the start of the scratch are zero when the device image is loaded and every launch
    // leaves them at zero; the kernels write every partial they later read.
    hipError_t e = launch_sparse_decode(desc->dtype, lp, pp, q, sel_pages, sel_count, sel_seq_len, sel_stride, out,
                                        lse_out, ws, (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

int lserve_probe_decode_read(const lserve_attn_desc* desc, const lserve_paged_kv* kv, const int32_t* sel_pages,
                             const int32_t* sel_count, const int32_t* sel_seq_len, int32_t sel_stride, void* stream) {
    LayerParams lp;
    PagedParams pp;
    int rc = make_layer(desc, &lp);
    if (rc) return rc;
    rc = make_paged(kv, lp, true, true, false, true, &pp);
    if (rc) return rc;
    const bool any_selecting = selecting_heads(lp).count > 0;
    if (any_selecting && (!sel_pages || !sel_count || !sel_seq_len || sel_stride <= 0)) return LSERVE_ERR_INVALID_ARG;
    if (sel_stride < 0 || !aligned16(sel_pages) || !aligned16(sel_count) || !aligned16(sel_seq_len)) return LSERVE_ERR_INVALID_ARG;
    if ((long long)pp.batch * lp.Hkv > 65535) return LSERVE_ERR_UNSUPPORTED;  // one grid row per (sequence, KV head)
    hipError_t e = launch_decode_read_probe(lp, pp, sel_pages, sel_count, sel_seq_len, sel_stride, (hipStream_t)stream);
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

size_t lserve_workspace_bytes(int which_call, const lserve_attn_desc* desc, int32_t batch, int32_t max_pages_per_seq,
                              int32_t sel_stride_or_budget_pages, int32_t total_tokens) {
    LayerParams lp;
    if (make_layer(desc, &lp) != LSERVE_OK) return 0;
    switch (which_call) {
        case LSERVE_CALL_SELECT_PAGES:
            return batch > 0 && max_pages_per_seq > 0 ? select_workspace_bytes(lp, batch, max_pages_per_seq) : 0;
        case LSERVE_CALL_SPARSE_PREFILL:
            return batch > 0 && total_tokens > 0 ? prefill_workspace_bytes(lp, total_tokens, batch) : 0;
        case LSERVE_CALL_SPARSE_DECODE:
            return batch > 0 && sel_stride_or_budget_pages >= 0
                       ? decode_workspace_bytes(lp, batch, sel_stride_or_budget_pages)
                       : 0;
        default:
            return 0;
    }
}

int lserve_init(void) {
    void* ws = nullptr;
    const int rc = scratch_on_current_device(&ws);
    if (rc) return rc;
    hipError_t e = preload_stats_kernels();
    if (e == hipSuccess) e = preload_select_kernels();
    if (e == hipSuccess) e = preload_prefill_kernels();
    if (e == hipSuccess) e = preload_decode_kernels();
    return e == hipSuccess ? LSERVE_OK : fail_hip(e);
}

const char* lserve_strerror(int code) {
    switch (code) {
        case LSERVE_OK:
            return "success";
        case LSERVE_ERR_INVALID_ARG:
            return "invalid argument (null or misaligned pointer, non-positive size, bad page sizes or budget)";
        case LSERVE_ERR_UNSUPPORTED:
            return "unsupported configuration (head_dim, dtype, head counts or page size)";
        case LSERVE_ERR_WORKSPACE:
            return "workspace missing or too small";
        case LSERVE_ERR_HIP:
            return "a HIP call failed (see lserve_last_hip_error)";
        default:
            return "unknown error code";
    }
}

int lserve_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
