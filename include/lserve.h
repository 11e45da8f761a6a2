/*
 * lserve.h -- C ABI of the unified block-sparse attention path of LServe (arxiv 2502.14866)
 * for AMD MI355X (gfx950).
 *
 * Four operations, one GPU, no hidden state:
 *   lserve_sparse_prefill    block-sparse causal prefill attention (Sec. 3.1, Sec. 3.4)
 *   lserve_build_page_stats  per-logical-page channel-wise key min / max (Sec. 3.5.2)
 *   lserve_select_pages      query-centric page scores (Eq. 2), max over logical pages,
 *                            top-K physical pages under a token budget (Sec. 3.5.2)
 *   lserve_sparse_decode     paged decode attention over an index table (Sec. 3.6)
 * and, around them, lserve_append_kv: write-back of new K/V into the pages with the statistics
 * updated in the same pass (Sec. 3.2, Sec. 3.5.2), lserve_sparse_prefill_masked: prefill under a
 * caller-supplied block mask (Sec. 3.1, Sec. 3.4), lserve_sparse_prefill_paged: chunked prefill whose keys
 * and values all come from the paged cache (Sec. 2.1), and lserve_sparse_prefill_chunk: chunked prefill over
 * the history in the cache with the chunk's own K / V alongside, before their write-back (Sec. 3.2).
 *
 * Conventions common to every call
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory.  The library allocates nothing, frees nothing and keeps no state that a result
 *     depends on.  What it does keep, per process, are properties of the GPU read on first use (the
 *     number of compute units of the device that is current at the first call, and for each decode
 *     kernel variant how many of its workgroups fit a compute unit); they fix the work split, so all
 *     calls of a process must run on GPUs of one kind.  No environment variable is read.
 *     Buffers are borrowed until the work enqueued by the call has completed on `stream`.
 *   - The first call that launches a kernel loads the library's code objects onto the device, which is
 *     not allowed while `stream` is being captured into a HIP graph: call lserve_init() (or run each
 *     entry point once eagerly) before capturing.  After that every call may be captured.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls validate their
 *     arguments on the host, enqueue kernels and return; they never synchronise.
 *   - Return value: LSERVE_OK (0) or a negative LSERVE_ERR_* code.  Nothing is printed, nothing
 *     aborts.  After LSERVE_ERR_HIP, lserve_last_hip_error() returns the hipError_t value.
 *   - Device-side data errors (a page id outside the pool, a sequence length of 0 or beyond
 *     max_pages_per_seq * page_size, a selected page >= the sequence's page count, duplicates in a
 *     selection) are not detected and give undefined results.
 *   - All device pointers must be 16-byte aligned.  Element type of Q/K/V/O/pools/stats is IEEE
 *     binary16 (dtype 0) or bfloat16 (dtype 1); accumulation is fp32.
 *   - Results are deterministic: the same inputs give bit-identical outputs (fixed reduction
 *     orders, no floating-point atomics).
 *
 * Symbols (paper notation): H query heads, Hkv KV heads, n = H / Hkv, D head dimension (128),
 * N_P tokens per physical page, N_L tokens per logical page, g = N_P / N_L, L_b current KV length
 * of sequence b, P_b = ceil(L_b / N_P), K = floor(budget / N_P).
 */
#ifndef LSERVE_H
#define LSERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LSERVE_OK 0
#define LSERVE_ERR_INVALID_ARG (-1) /* null / misaligned pointer, non-positive size, bad page sizes, budget < N_P */
#define LSERVE_ERR_UNSUPPORTED (-2) /* head_dim != 128, unknown dtype, H % Hkv != 0, Hkv > 64, n > 8, g > 8, batch > 65535 */
#define LSERVE_ERR_WORKSPACE (-3)   /* workspace missing or smaller than lserve_workspace_bytes() */
#define LSERVE_ERR_HIP (-4)         /* a HIP call failed; see lserve_last_hip_error() */

#define LSERVE_DTYPE_FP16 0
#define LSERVE_DTYPE_BF16 1

/* which_call values for lserve_workspace_bytes() */
#define LSERVE_CALL_BUILD_PAGE_STATS 0
#define LSERVE_CALL_SELECT_PAGES 1
#define LSERVE_CALL_SPARSE_PREFILL 2
#define LSERVE_CALL_SPARSE_DECODE 3

/*
 * Attention layer description (Sec. 2.1 for H, Hkv, D; Sec. 3.1 for streaming heads and their
 * sink / local sizes; Sec. 3.5.2 for N_P and N_L).
 *
 * The streaming pattern is tile granular (Sec. 3.1: a tile is kept whole or skipped whole):
 * s = ceil(sink_tokens / N_P) leading tiles and w = ceil(local_tokens / N_P) trailing tiles,
 * the query's own tile included, are kept; inside kept tiles only causality masks.  The prefill
 * mask tile and the decode page are both N_P tokens, so prefill row t and a decode step at
 * length t + 1 attend the same tokens.
 */
typedef struct lserve_attn_desc {
    int32_t num_q_heads;       /* H */
    int32_t num_kv_heads;      /* Hkv, H % Hkv == 0, Hkv <= 64, H / Hkv <= 8 */
    int32_t head_dim;          /* D, must be 128 */
    int32_t page_size;         /* N_P: 16, 32, 64 or 128; prefill requires 64 */
    int32_t logical_page_size; /* N_L: divides N_P, N_P / N_L <= 8, N_L >= 1 */
    int32_t dtype;             /* LSERVE_DTYPE_* */
    int32_t sink_tokens;       /* >= 0, rounded up to whole tiles */
    int32_t local_tokens;      /* >= 1, rounded up to whole tiles */
    const uint8_t *kv_head_is_streaming; /* HOST, [Hkv], 1 = streaming head, 0 = dense / selecting head */
    float sm_scale;            /* softmax scale; 0 means 1 / sqrt(D) */
} lserve_attn_desc;

/*
 * Paged KV cache (Sec. 2.1 "Paged Attention"; Sec. 3.5.2 for the statistics; Sec. 3.2 for the
 * two-way cache).
 * Token t of sequence b is slot t % N_P of physical page page_table[b][t / N_P].
 *
 * One pool (pool_heads == 0 or Hkv, k_pool_stream == NULL): every KV head lives in k_pool / v_pool.
 *
 * Two-way cache (Sec. 3.2: dense heads and streaming heads keep separate caches, the streaming one
 * holding only sink and local tokens): set pool_heads to the number of non-streaming KV heads; k_pool,
 * v_pool and stats then hold only those heads, in KV-head order.  Streaming heads live in
 * k_pool_stream / v_pool_stream, [num_pages_stream][Hs][N_P][D] with Hs the number of streaming heads
 * (KV-head order), through a ring of s + w pages per sequence: the page at position p of the sequence
 * (p = t / N_P) is ring slot r(p) = p for p < s, s + (p - s) % w otherwise, stored in physical page
 * ring_table[b][r(p)].  A local page is overwritten by the page w positions later, so at length L_b
 * only pages p < s and p >= P_b - w are present, which is all a streaming head attends (Sec. 3.1).
 * k_pool_stream may also be given next to a main pool that holds every head (pool_heads == Hkv):
 * the streaming heads are then read from and written to the ring only.
 *
 * Quantised pages (kv_bits == 8 or 4; Sec. 3.2: scale factors and zero points are stored right after the
 * token features; Sec. 3.5: low-bit KV is why the physical page is 64 tokens).  Requires N_P == 64.  Every
 * pool then stores, per (page, head), 64 rows of D codes of kv_bits bits followed by 64 pairs (scale, zero)
 * of fp16, 64 * D * kv_bits / 8 + 256 bytes in all, and a stored row stands for code * scale + zero.  8-bit
 * rows hold channel c in byte c.  4-bit rows are D / 8 words of four bytes, byte j of word g holding channel
 * 8 g + j in its low half and channel 8 g + 4 + j in its high half.  The quantiser is per token and per KV
 * head, separately for K and V, with top = 2^kv_bits - 1:
 *     zero = fp16(min_c x_c), scale = fp16((max_c x_c - zero) / top),
 *     code_c = clamp(rint((x_c - zero) / scale), 0, top), all codes 0 when scale == 0,
 * in IEEE fp32 with round to nearest even (fp16 conversions saturate at 65504).  lserve_append_kv writes
 * such pages (statistics are taken from the 16-bit keys it is handed) and lserve_sparse_decode reads them;
 * lserve_select_pages works from the statistics alone, so only its rebuild of stale statistics
 * (stats_valid_len) is unavailable; lserve_sparse_prefill_chunk reads them as the history of a chunk;
 * lserve_build_page_stats and lserve_sparse_prefill_paged return LSERVE_ERR_UNSUPPORTED.  The stats array keeps the
 * 16-bit layout.
 */
typedef struct lserve_paged_kv {
    void *k_pool;              /* device, [num_pages][pool_heads][N_P][D]; quantised: [num_pages][pool_heads][64 * D * kv_bits / 8 + 256] bytes */
    void *v_pool;              /* device, same shape as k_pool */
    void *stats;               /* device, [num_pages][pool_heads][g][2][D]; [..][0][:] = max, [..][1][:] = min */
    const int32_t *page_table; /* device, [batch][max_pages_per_seq], physical page ids in [0, num_pages) */
    const int32_t *seq_lens;   /* device, [batch], 1 <= L_b <= max_pages_per_seq * N_P */
    int32_t batch;
    int32_t max_pages_per_seq;
    int32_t num_pages;
    int32_t pool_heads;        /* 0 = Hkv; otherwise Hkv or the number of non-streaming KV heads */
    void *k_pool_stream;       /* device, [num_pages_stream][Hs][N_P][D], or NULL */
    void *v_pool_stream;       /* device, same shape, or NULL (both or neither) */
    const int32_t *ring_table; /* device, [batch][s + w], page ids in [0, num_pages_stream) */
    int32_t num_pages_stream;
    int32_t kv_bits;           /* 0 or 16: K/V rows in the 16-bit dtype of the layer; 8 or 4: quantised pages */
} lserve_paged_kv;

/*
 * Key statistics (Sec. 3.5.2; caption of the hierarchical-paging figure): for every non-streaming
 * KV head, every logical page that overlaps tokens [start_pos[b], L_b) of sequence b and every
 * channel c, write max and min of K[t][c] over the page's valid tokens t < L_b into kv->stats.
 * Statistics of logical pages without a valid token are not written.
 *
 *   start_pos      device [batch] or NULL (= 0 for every sequence: full rebuild after prefill).
 *                  After appending one token call with start_pos[b] = L_b - 1.
 *   max_tail_pages host hint: no sequence has more than this many physical pages overlapping
 *                  [start_pos, L_b); 0 = unknown (all max_pages_per_seq are visited).  A too small
 *                  hint leaves the oldest pages of the range stale.
 * Reads kv->k_pool, page_table, seq_lens; writes kv->stats.  No workspace.
 */
int lserve_build_page_stats(const lserve_attn_desc *desc, const lserve_paged_kv *kv,
                            const int32_t *start_pos, int32_t max_tail_pages, void *stream);

/*
 * KV write-back with fused statistics (Sec. 3.2: prefill writes K/V back into the paged cache; Sec. 3.5.2
 * and the caption of the hierarchical-paging figure: the statistics are computed during the context
 * stage and the previous decoding steps).  Appends n_b = cu_new[b+1] - cu_new[b] tokens to every
 * sequence: new token j of sequence b is stored at position start_pos[b] + j, i.e. slot
 * (start_pos[b] + j) % N_P of physical page page_table[b][(start_pos[b] + j) / N_P], for every KV head,
 * in both pools.  For non-streaming KV heads the max / min rows of every logical page that received a
 * token are brought up to date without re-reading old keys: a logical page that already held tokens
 * (positions below start_pos[b]) combines its stored statistics with the new keys, which requires
 * kv->stats to be current for positions below start_pos[b]; a logical page whose first token is new
 * is computed from the new keys alone.  kv->seq_lens must be a valid pointer as in every call but is
 * neither read nor written (the caller bumps the lengths).  kv->stats may be NULL when every KV head is
 * streaming.  With kv->kv_bits == 8 or 4 the rows are quantised on the way in (see lserve_paged_kv: one
 * scale and zero point per token, KV head and pool, written behind the page's rows); the statistics are
 * those of the 16-bit keys handed in, exactly as for a 16-bit cache.
 *
 *   k_new, v_new   device [total_new][Hkv][D], tokens of all sequences concatenated
 *   cu_new         device [batch + 1], cu_new[0] = 0
 *   start_pos      device [batch]; start_pos[b] + n_b <= max_pages_per_seq * N_P
 *   max_new_per_seq  host upper bound of n_b (sizes the launch); > 0
 * Reads page_table, k_new, v_new, stats; writes k_pool, v_pool, stats.  No workspace.
 */
int lserve_append_kv(const lserve_attn_desc *desc, const lserve_paged_kv *kv, const void *k_new,
                     const void *v_new, const int32_t *cu_new, const int32_t *start_pos,
                     int32_t max_new_per_seq, void *stream);

/*
 * Page selection (Eq. 2 and the paragraph after it; Sec. 3.2 "shorter page tables").
 * For every sequence b and non-streaming KV head hk:
 *   logical page score  S_h^l = sum_c max(q_h[c] * kmax^l[c], q_h[c] * kmin^l[c])   (no 1/sqrt(D)),
 *   group score         = max over the n query heads h of KV head hk,
 *   physical page score = max over the page's logical pages that hold a valid token,
 *   selection           = all P_b pages if P_b <= K, else page P_b - 1 (newest token) plus the
 *                         K - 1 best-scoring other pages, a tie going to the lower page index.
 * Scores are accumulated in fp32 in a fixed order.
 *
 *   q            device [batch][H][D]
 *   budget_tokens  K = budget_tokens / N_P, must be >= 1
 *   stats_valid_len  device [batch] or NULL.  NULL: kv->stats is current for every token below L_b.
 *                Otherwise kv->stats is current only for tokens below stats_valid_len[b] (<= L_b):
 *                the logical pages that hold tokens [stats_valid_len[b], L_b) are recomputed from
 *                kv->k_pool inside this call (Sec. 3.5.2: statistics of the tokens decoded since the
 *                last selection), used for the scores and written back to kv->stats, which saves the
 *                separate lserve_build_page_stats launch in a decode loop.  Needs kv->k_pool.
 *   sel_pages    device [batch][Hkv][K] out: positions of the selected pages inside the sequence
 *                (indices into page_table[b]), ascending; entries past sel_count are -1.
 *                Rows of streaming heads are filled with -1.
 *   sel_count    device [batch][Hkv] out (0 for streaming heads)
 *   sel_seq_len  device [batch] out: L_b at selection time
 *   scores_out   device [batch][Hkv][max_pages_per_seq] fp32 or NULL: physical page scores
 *                (entries p >= P_b and rows of streaming heads are 0)
 *   workspace    device, >= lserve_workspace_bytes(LSERVE_CALL_SELECT_PAGES, ...)
 */
int lserve_select_pages(const lserve_attn_desc *desc, const lserve_paged_kv *kv, const void *q,
                        int32_t budget_tokens, const int32_t *stats_valid_len, int32_t *sel_pages,
                        int32_t *sel_count, int32_t *sel_seq_len, float *scores_out, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * Block-sparse causal prefill (Eq. 1 under the block mask of Sec. 3.1; Sec. 3.4).
 * Tokens of all sequences are concatenated.  For the token at position t of its sequence and
 * query head h (KV head h / n), the allowed keys are the positions u <= t of the same sequence
 * with, for a streaming head, tile(u) < s or tile(u) > tile(t) - w, tile(x) = x / 64.
 * out = softmax(scale * q . k_u over allowed u) applied to v_u; tiles with no allowed pair are
 * never loaded.
 *
 *   q            device [total_tokens][H][D]
 *   k, v         device [total_tokens][Hkv][D]
 *   cu_seqlens   device [batch + 1], cu_seqlens[0] = 0, cu_seqlens[batch] = total_tokens
 *   max_seqlen   host: upper bound of the sequence lengths (sizes the launch)
 *   out          device [total_tokens][H][D]
 *   lse_out      device [H][total_tokens] fp32 or NULL: natural-log sum of exp of the scaled scores
 *   workspace    unused: lserve_workspace_bytes(LSERVE_CALL_SPARSE_PREFILL, ...) is 0 (Q, K and V are read where
 *                they are); NULL is accepted
 * Requires desc->page_size == 64 (the mask tile).
 */
int lserve_sparse_prefill(const lserve_attn_desc *desc, const void *q, const void *k, const void *v,
                          const int32_t *cu_seqlens, int32_t batch, int32_t total_tokens,
                          int32_t max_seqlen, void *out, float *lse_out, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Chunked prefill over the paged cache (Sec. 2.1: prefill of N tokens with S tokens of KV history; mask of
 * Sec. 3.1).  The K / V of every token, the chunk's own included (lserve_append_kv first), are read from
 * kv; sequence b has L_b = kv->seq_lens[b] tokens and the chunk is its last n_b = cu_q[b+1] - cu_q[b]
 * tokens, so query j sits at position t = L_b - n_b + j and attends the positions u <= t that the analytic
 * mask of `desc` allows, tiles counted from position 0.  With n_b = L_b this equals lserve_sparse_prefill on
 * the same tokens; with n_b = 1 it equals a decode step with nothing left out for dense heads.
 *
 *   kv           one pool holding every KV head (pool_heads 0 or Hkv, no streaming pool), N_P = 64;
 *                stats are not used
 *   q            device [total_new][H][D], cu_q device [batch + 1] (batch = kv->batch), n_b >= 0
 *   max_new_per_seq  host bound of n_b (> 0); max_seqlen host bound of L_b
 *   out          device [total_new][H][D]; lse_out device [H][total_new] fp32 or NULL
 *   workspace    unused: lserve_paged_prefill_workspace_bytes() is 0 (keys and values are read from the pages as
 *                they are); NULL is accepted
 */
int lserve_sparse_prefill_paged(const lserve_attn_desc *desc, const lserve_paged_kv *kv, const void *q,
                                const int32_t *cu_q, int32_t total_new, int32_t max_new_per_seq,
                                int32_t max_seqlen, void *out, float *lse_out, void *workspace,
                                size_t workspace_bytes, void *stream);

size_t lserve_paged_prefill_workspace_bytes(const lserve_attn_desc *desc, int32_t batch,
                                            int32_t max_pages_per_seq);

/*
 * Chunked prefill in the order of the prefill flow (Sec. 3.2: attention over the new tokens first, then their K / V
 * are written back into the two caches; Sec. 2.1: N new tokens with S tokens of KV history; mask of Sec. 3.1).
 * Sequence b has S_b = kv->seq_lens[b] tokens of history in the cache (S_b >= 0 here) and n_b = cu_new[b+1] - cu_new[b]
 * new tokens whose Q, K and V arrive contiguously.  Query j sits at position t = S_b + j and attends the positions
 * u <= t that the analytic mask of `desc` allows, tiles counted from position 0: keys u < S_b are read from the cache,
 * keys u >= S_b from k_new / v_new.  Nothing is written to the cache: call lserve_append_kv with the same k_new, v_new,
 * cu_new (and start_pos = the lengths) afterwards.  With S_b = 0 everywhere this equals lserve_sparse_prefill.
 *
 *   kv           the history, N_P = 64: one pool holding every KV head, or the two-way cache (dense heads in the
 *                main pool, streaming heads in their ring: the ring of a sequence of S_b tokens holds the sink pages
 *                and the last w pages, which is every history key a streaming query of the chunk may attend; the keys
 *                between come from the chunk itself).  Pages of 16-bit rows or quantised pages (kv_bits 8 or 4): a
 *                history key / value is then the number its code stands for, code * scale + zero, computed in fp32
 *                and rounded to the layer's 16-bit type on its way to the matrix cores.  stats are not used.
 *   q            device [total_new][H][D]; k_new, v_new device [total_new][Hkv][D]
 *   cu_new       device [batch + 1] (batch = kv->batch), cu_new[0] = 0, n_b >= 0
 *   max_new_per_seq  host bound of n_b (> 0)
 *   out          device [total_new][H][D]; lse_out device [H][total_new] fp32 or NULL
 * No workspace.
 */
int lserve_sparse_prefill_chunk(const lserve_attn_desc *desc, const lserve_paged_kv *kv, const void *q,
                                const void *k_new, const void *v_new, const int32_t *cu_new, int32_t total_new,
                                int32_t max_new_per_seq, void *out, float *lse_out, void *stream);

/*
 * Block-sparse prefill under a general block mask (Sec. 3.1: every tile of the attention map is skipped or
 * computed whole; Sec. 3.4: the kernel walks whatever list of key tiles it is given, the analytic
 * streaming pattern being one case).  A mask lists, for every 64-row query tile i of every sequence, the
 * 64-key tiles it keeps, in CSR form; query head h uses mask head_mask[h], or the analytic mask of `desc`
 * (dense or streaming, as in lserve_sparse_prefill) when head_mask[h] = -1.  Key u is attended by query t
 * iff u <= t and tile(u) is listed in the row of tile(t); the diagonal tile, if listed, is causal inside.
 * A query row whose tile row lists nothing gets out = 0 and lse = -inf.
 *
 *   head_mask      device [H], values in [-1, num_masks)
 *   q_tile_start   device [batch + 1]: row of query tile 0 of sequence b inside one mask;
 *                  q_tile_start[b + 1] - q_tile_start[b] = ceil(len_b / 64), q_tile_start[batch] = rows_per_mask
 *   row_ptr        device [num_masks * rows_per_mask + 1]; row of (mask m, sequence b, tile i) is
 *                  r = m * rows_per_mask + q_tile_start[b] + i, its entries cols[row_ptr[r] .. row_ptr[r + 1])
 *   cols           device [nnz]: key tile indices inside the sequence, strictly ascending within a row;
 *                  entries above the row's own tile index are ignored
 *   workspace      device, >= lserve_masked_prefill_workspace_bytes(...)
 * Other arguments as in lserve_sparse_prefill.  Data errors inside the CSR arrays (unsorted rows, row_ptr
 * not monotone or beyond nnz) are not detected.  Unsupported: max_seqlen > 4194304.
 */
typedef struct lserve_block_mask {
    const int32_t *head_mask;
    const int32_t *q_tile_start;
    const int32_t *row_ptr;
    const int32_t *cols;
    int32_t num_masks;
    int32_t rows_per_mask;
    int32_t nnz;
} lserve_block_mask;

int lserve_sparse_prefill_masked(const lserve_attn_desc *desc, const lserve_block_mask *mask, const void *q,
                                 const void *k, const void *v, const int32_t *cu_seqlens, int32_t batch,
                                 int32_t total_tokens, int32_t max_seqlen, void *out, float *lse_out,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* Workspace of lserve_sparse_prefill_masked (0 on invalid arguments). */
size_t lserve_masked_prefill_workspace_bytes(const lserve_attn_desc *desc, int32_t batch, int32_t total_tokens,
                                             int32_t max_seqlen, int32_t num_masks, int32_t nnz);

/*
 * Paged sparse decode (Eq. 1 over the pages of an index table; Sec. 3.6).
 * One query token per sequence; its K/V are already in the pool and counted in L_b.
 * Page list of KV head hk:
 *   streaming head: pages p < s and pages p > P_b - 1 - w (sink and local pages, each once);
 *                   its rows of sel_pages / sel_count are ignored;
 *   selecting head: sel_pages[b][hk][0 .. sel_count) followed by every page
 *                   p >= ceil(sel_seq_len[b] / N_P), i.e. pages created since the selection
 *                   (reusable page selection, Sec. 3.5.3).
 * All n query heads of the group attend the valid tokens (u < L_b) of the listed pages.
 * Over quantised pages (kv->kv_bits == 8 or 4) the keys and values are the numbers the stored codes stand
 * for, code * scale + zero; the queries are then taken in fp16 (a bf16 query beyond 65504 in magnitude
 * saturates).
 *
 *   q            device [batch][H][D]
 *   sel_pages    device [batch][Hkv][sel_stride], sel_count device [batch][Hkv],
 *   sel_seq_len  device [batch]; all three may be NULL when every KV head is streaming
 *   out          device [batch][H][D]
 *   lse_out      device [batch][H] fp32 or NULL
 *   workspace    device, >= lserve_workspace_bytes(LSERVE_CALL_SPARSE_DECODE, ...).  It must be zero-filled once
 *                before the first call that uses it (it starts with one arrival counter per (sequence, KV head)
 *                list, which every call leaves at zero again); after that it may go from call to call, also
 *                between different shapes that fit it.  Two calls that may run at the same time need a workspace each.
 * LSERVE_ERR_UNSUPPORTED when batch * (index-table entries per sequence) exceeds 2^31 - 1, an entry count
 * being s + w per streaming head and sel_stride + 1 per selecting head.
 */
int lserve_sparse_decode(const lserve_attn_desc *desc, const lserve_paged_kv *kv, const void *q,
                         const int32_t *sel_pages, const int32_t *sel_count,
                         const int32_t *sel_seq_len, int32_t sel_stride, void *out, float *lse_out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * lserve_sparse_decode for callers that cannot allocate device memory (code under HIP graph capture, serving
 * loops and harnesses that forbid hipMalloc) and so have no workspace to hand over: the partial results go to a
 * fixed scratch array of LSERVE_NOALLOC_SCRATCH_BYTES inside the library's device image, one copy per GPU, held
 * until the process ends.  Same arguments, same kernels and bit-identical results as lserve_sparse_decode, minus
 * the workspace.  Neither this call nor anything it uses allocates or frees memory.
 *   - LSERVE_ERR_WORKSPACE when lserve_workspace_bytes(LSERVE_CALL_SPARSE_DECODE, ...) for these arguments exceeds
 *     LSERVE_NOALLOC_SCRATCH_BYTES (on a 256-CU device with n = 4: batch * Hkv > 3008 lists); every other error as
 *     in lserve_sparse_decode.
 *   - All calls on one GPU share that GPU's scratch: two calls whose kernels may run at the same time on one GPU
 *     (different streams, different threads) race and give undefined results; calls ordered on one stream are fine.
 *     The scratch keeps the last call's partials; each call writes every slot it reads and leaves the arrival
 *     counters at its start at zero, which is how the device image initialises them: nothing has to be cleared.
 *   - The address of the scratch is resolved once per device, at lserve_init() or at the first call on that device
 *     (with that device current).  Call lserve_init() before capturing a stream if the first call would otherwise
 *     happen under capture.
 */
#define LSERVE_NOALLOC_SCRATCH_BYTES (8u << 20)
int lserve_sparse_decode_noalloc(const lserve_attn_desc *desc, const lserve_paged_kv *kv, const void *q,
                                 const int32_t *sel_pages, const int32_t *sel_count,
                                 const int32_t *sel_seq_len, int32_t sel_stride, void *out, float *lse_out,
                                 void *stream);

/*
 * Measurement aid, not part of the attention path (Sec. 3.6 defines what the decode call reads): issues the reads
 * of lserve_sparse_decode for the same arguments (the K and V slabs of every page the index tables of the batch
 * list, through the same page tables) from one short workgroup per table entry, and discards the data.  Nothing
 * is written.  Its duration is what the memory system charges for the decode call's access pattern alone; bench.py
 * reports it next to the call.  Lists are read up to their nominal length plus eight pages created since the
 * selection.  Arguments and errors as for lserve_sparse_decode, without q, out, lse_out and workspace;
 * LSERVE_ERR_UNSUPPORTED for more than 65535 (sequence, KV head) lists.
 */
int lserve_probe_decode_read(const lserve_attn_desc *desc, const lserve_paged_kv *kv, const int32_t *sel_pages,
                             const int32_t *sel_count, const int32_t *sel_seq_len, int32_t sel_stride,
                             void *stream);

/*
 * Bytes of device workspace a call needs (Sec. 3.6 / 3.5.2 calls keep partial results there).
 *   batch, max_pages_per_seq: as in lserve_paged_kv (ignored for prefill)
 *   sel_stride_or_budget_pages: K for select, sel_stride for decode (ignored otherwise)
 *   total_tokens: prefill only
 * Returns 0 when the call needs none or when desc is invalid.
 */
size_t lserve_workspace_bytes(int which_call, const lserve_attn_desc *desc, int32_t batch,
                              int32_t max_pages_per_seq, int32_t sel_stride_or_budget_pages,
                              int32_t total_tokens);

/*
 * Optional set-up for the device that is current on the calling thread: loads the library's code objects
 * onto it, so that later calls do no loading and may run under stream capture.  Safe to call more than once and
 * from several threads; launches nothing.  Returns LSERVE_OK or LSERVE_ERR_HIP.
 */
int lserve_init(void);

/* Human-readable text for a return code (static storage). */
const char *lserve_strerror(int code);

/* hipError_t of the last failed HIP call on the calling thread (0 if none). */
int lserve_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LSERVE_H */
