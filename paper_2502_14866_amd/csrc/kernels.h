// Host-visible launchers of the gfx950 kernels.  The C ABI (lserve_api.hip) validates arguments
// and calls these; each returns the hipError_t of its launch.
#pragma once

#include "common.h"

namespace lserve {

// Compact list of KV head indices (e.g. the non-streaming heads), passed by value to kernels.
struct HeadList {
    int count;
    unsigned char idx[64];
};

hipError_t launch_page_stats(int dtype, const LayerParams& lp, const PagedParams& kv, const int* start_pos,
                             int tail_pages, const HeadList& heads, hipStream_t stream);

hipError_t launch_append_kv(int dtype, const LayerParams& lp, const PagedParams& kv, const void* k_new, const void* v_new,
                            const int* cu_new, const int* start_pos, int max_new_per_seq, hipStream_t stream);

hipError_t launch_select_pages(int dtype, const LayerParams& lp, const PagedParams& kv, const void* q,
                               const int* stats_valid_len, int budget_pages, int* sel_pages, int* sel_count, int* sel_seq_len,
                               float* scores, bool scores_is_user_buffer, const HeadList& selecting,
                               hipStream_t stream);

size_t paged_prefill_workspace_bytes(const LayerParams& lp, int batch, int max_pages);
// k_new / v_new: the chunk's own K / V when they have not been written back yet (the cache is then the chunk's
// history), or null when the cache already holds the chunk.
hipError_t launch_sparse_prefill_paged(int dtype, const LayerParams& lp, const PagedParams& kv, const void* q,
                                       const void* k_new, const void* v_new, const int* cu_q, int total_new,
                                       int max_new_per_seq, int max_seqlen, void* out, float* lse_out, void* workspace,
                                       hipStream_t stream);

size_t decode_workspace_bytes(const LayerParams& lp, int batch, int sel_stride);

// Nominal index-table entries per sequence of a decode launch: s + w per streaming head, sel_stride + 1 per
// selecting head.  The launch plan indexes batch * this many entries with 32-bit integers.
long long decode_nominal_entries(const LayerParams& lp, int sel_stride);

// Each forces the code object of its translation unit onto the current device (HIP loads them on first use).
hipError_t preload_decode_kernels();
hipError_t preload_select_kernels();
hipError_t preload_stats_kernels();
hipError_t preload_prefill_kernels();

hipError_t launch_sparse_decode(int dtype, const LayerParams& lp, const PagedParams& kv, const void* q,
                                const int* sel_pages, const int* sel_count, const int* sel_seq_len,
                                int sel_stride, void* out, float* lse_out, void* workspace, hipStream_t stream);

// measurement aid: reads what the decode call above would read and discards it
hipError_t launch_decode_read_probe(const LayerParams& lp, const PagedParams& kv, const int* sel_pages, const int* sel_count,
                                    const int* sel_seq_len, int sel_stride, hipStream_t stream);

// Caller-side description of a general block mask for prefill (device pointers).
struct PrefillMaskArgs {
    const int* head_mask;
    const int* q_tile_start;
    const int* row_ptr;
    const int* cols;
    int num_masks, rows_per_mask, nnz;
};

size_t prefill_workspace_bytes(const LayerParams& lp, int total_tokens, int batch);
size_t masked_prefill_workspace_bytes(const LayerParams& lp, int total_tokens, int batch, int max_seqlen, int num_masks,
                                      int nnz);

hipError_t launch_sparse_prefill(int dtype, const LayerParams& lp, const void* q, const void* k, const void* v,
                                 const int* cu_seqlens, int batch, int total_tokens, int max_seqlen, void* out,
                                 float* lse_out, void* workspace, const PrefillMaskArgs* mask, hipStream_t stream);

}  // namespace lserve
