/*
 * CPU oracle for the unified block-sparse attention path (LServe, arxiv 2502.14866).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * GPU library must compute.  It is used by the tests, by the smoke check and by
 * the CPU-baseline leg of the benchmark.  The product path never calls it, and it
 * shares no code, header, table or helper with the HIP sources.
 *
 * Everything is written straight from the definitions, in double precision, with
 * no tiling, fusion or reordering:
 *   - attention                      : Eq. 1 (Sec. 2.1), restricted to an allowed key set
 *   - block sparsity / streaming mask: Sec. 3.1 (tiles are kept or skipped whole; streaming
 *                                      heads keep sink tiles and a local band)
 *   - key statistics                 : Sec. 3.5.2 and the hierarchical-paging figure caption
 *                                      (channel-wise min / max of the keys of a logical page)
 *   - logical page importance        : Eq. 2 (Sec. 3.5.2)
 *   - physical page importance, top-K: Sec. 3.5.2 last paragraph (max over logical pages,
 *                                      K highest pages under the token budget)
 *   - decode over an index table     : Sec. 3.6 (selected pages for dense heads, sink + local
 *                                      pages for streaming heads), Sec. 3.2 ("shorter page table")
 *   - chunked prefill over paged KV  : Sec. 2.1 (prefill with S tokens of history), mask of Sec. 3.1; also in the
 *                                      order of the prefill flow of Sec. 3.2 (history from the cache, the chunk's
 *                                      own K / V not yet written back)
 *   - general block mask in prefill  : Sec. 3.1 / Sec. 3.4 (kept key tiles listed per query tile and head)
 *   - KV write-back                  : Sec. 3.2 / Sec. 2.1 (new tokens stored at their slots of the
 *                                      paged cache; statistics afterwards = the definition above
 *                                      evaluated at the new lengths)
 *
 * Readings taken where the paper is silent (the same ones bind the GPU path):
 *   - the streaming mask is tile granular: s = ceil(sink / T) sink tiles and w = ceil(local / T)
 *     local tiles counting the diagonal tile; inside kept tiles only causality masks;
 *   - under grouped-query attention there is one selection per KV head and the score of a
 *     logical page is the maximum of Eq. 2 over the query heads of the group;
 *   - the page that holds the newest token is always selected and counts inside K; ties go to
 *     the lower page index; the selected list is ascending;
 *   - decode with a reused selection also attends every page created after the selection;
 *   - logical pages without a valid token are ignored; statistics cover valid tokens only;
 *   - scores carry no 1/sqrt(D) factor.
 *
 * Parity pins for every function here live in tests/test_oracle_*.py.  The paper prints no
 * worked numeric example of scores, selections or outputs, so the whole path against the
 * paper's own numbers is "parity unpinned"; each function is pinned against closed forms,
 * brute force, invariants and library routines instead.
 *
 * Storage dtypes: 0 = IEEE binary16, 1 = bfloat16, both passed as raw 16-bit patterns.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- exact widening of 16-bit floats ------------------------------------------------ */

double oracle_widen(uint16_t bits, int dtype)
{
    if (dtype == 1) { /* bfloat16 is the upper half of a binary32 */
        uint32_t u = ((uint32_t)bits) << 16;
        float f;
        memcpy(&f, &u, sizeof f);
        return (double)f;
    }
    int sign = (bits >> 15) & 1;
    int expo = (bits >> 10) & 0x1f;
    int frac = bits & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24); /* subnormal: frac * 2^-10 * 2^-14 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

/* Element (token slot t, channel c) of KV head hk in physical page `page` of a pool laid out
 * [num_pages][Hkv][N_P][D]. */
static inline size_t pool_index(int page, int hk, int t, int c, int Hkv, int NP, int D)
{
    return (((size_t)page * Hkv + hk) * NP + t) * D + c;
}

/* ---- key statistics (Sec. 3.5.2; hierarchical-paging figure caption) ------------------ */
/*
 * For sequence b, KV head hk, logical page l = tokens [l*NL, (l+1)*NL) below seq_len, channel c:
 *   kmax[c] = max_t K[t][c],  kmin[c] = min_t K[t][c].
 * Token t lives in physical page page_table[b][t / NP], slot t % NP.
 * stats is [num_pages][Hkv][g][2][D] (index 0 = max, 1 = min), in the storage dtype; a minimum
 * or maximum of stored values is itself a stored value, so the bit pattern is written.
 * Entries of logical pages with no valid token are left untouched.
 */
void oracle_page_stats(const uint16_t *k_pool, const int32_t *page_table, const int32_t *seq_lens,
                       int batch, int max_pages, int Hkv, int D, int NP, int NL, int dtype,
                       uint16_t *stats)
{
    int g = NP / NL;
    for (int b = 0; b < batch; ++b) {
        int L = seq_lens[b];
        int n_logical = ceil_div(L, NL);
#pragma omp parallel for schedule(static)
        for (int l = 0; l < n_logical; ++l) {
            int t0 = l * NL;
            int t1 = t0 + NL < L ? t0 + NL : L;
            int page = page_table[(size_t)b * max_pages + t0 / NP];
            int j = (t0 % NP) / NL; /* logical page inside its physical page */
            for (int hk = 0; hk < Hkv; ++hk) {
                for (int c = 0; c < D; ++c) {
                    uint16_t bmax = 0, bmin = 0;
                    double vmax = 0.0, vmin = 0.0;
                    for (int t = t0; t < t1; ++t) {
                        uint16_t bits = k_pool[pool_index(page, hk, t % NP, c, Hkv, NP, D)];
                        double x = oracle_widen(bits, dtype);
                        if (t == t0 || x > vmax) { vmax = x; bmax = bits; }
                        if (t == t0 || x < vmin) { vmin = x; bmin = bits; }
                    }
                    size_t base = ((((size_t)page * Hkv + hk) * g + j) * 2) * D;
                    stats[base + c] = bmax;
                    stats[base + D + c] = bmin;
                }
            }
        }
    }
}

/* ---- KV write-back (Sec. 3.2; Sec. 2.1 "Paged Attention") -------------------------------- */
/*
 * Append n_b = cu_new[b+1] - cu_new[b] tokens to sequence b: new token j takes position
 * start_pos[b] + j, which is slot (position % NP) of physical page page_table[b][position / NP],
 * for every KV head, in both pools.  k_new / v_new are [total_new][Hkv][D].  Bit patterns are moved
 * unchanged.  Statistics are not touched here: the definition of the statistics after an append
 * is oracle_page_stats at the new lengths.
 */
void oracle_append_kv(const uint16_t *k_new, const uint16_t *v_new, const int32_t *cu_new,
                      const int32_t *start_pos, const int32_t *page_table, int batch, int max_pages,
                      int Hkv, int D, int NP, uint16_t *k_pool, uint16_t *v_pool)
{
    for (int b = 0; b < batch; ++b) {
        int n = cu_new[b + 1] - cu_new[b];
        for (int j = 0; j < n; ++j) {
            int pos = start_pos[b] + j;
            int page = page_table[(size_t)b * max_pages + pos / NP];
            for (int hk = 0; hk < Hkv; ++hk) {
                for (int c = 0; c < D; ++c) {
                    size_t src = (((size_t)(cu_new[b] + j)) * Hkv + hk) * D + c;
                    size_t dst = pool_index(page, hk, pos % NP, c, Hkv, NP, D);
                    k_pool[dst] = k_new[src];
                    v_pool[dst] = v_new[src];
                }
            }
        }
    }
}

/* ---- page importance (Eq. 2; Sec. 3.5.2 last paragraph) ------------------------------- */
/*
 * Logical page score of query head h:  S_h^l = sum_c max(q_h[c]*kmax^l[c], q_h[c]*kmin^l[c]).
 * KV-head score of a logical page      = max over the query heads h of the group of hk.
 * Physical page score                  = max over its logical pages that hold a valid token.
 * page_scores is [batch][Hkv][max_pages]; entries p >= ceil(L/NP) are set to 0.
 * logical_scores (may be NULL) is [batch][H][max_pages][g]; empty logical pages get 0.
 */
void oracle_page_scores(const uint16_t *q, const uint16_t *stats, const int32_t *page_table,
                        const int32_t *seq_lens, int batch, int max_pages, int H, int Hkv, int D,
                        int NP, int NL, int dtype, double *page_scores, double *logical_scores)
{
    int g = NP / NL;
    int n = H / Hkv;
    for (int b = 0; b < batch; ++b) {
        int L = seq_lens[b];
        int P = ceil_div(L, NP);
#pragma omp parallel for schedule(static)
        for (int p = 0; p < max_pages; ++p) {
            for (int hk = 0; hk < Hkv; ++hk) {
                double *dst = &page_scores[((size_t)b * Hkv + hk) * max_pages + p];
                *dst = 0.0;
                if (p >= P)
                    continue;
                int page = page_table[(size_t)b * max_pages + p];
                int have = 0;
                double best = 0.0;
                for (int j = 0; j < g; ++j) {
                    if (p * NP + j * NL >= L)
                        continue; /* logical page without a valid token */
                    size_t base = ((((size_t)page * Hkv + hk) * g + j) * 2) * D;
                    for (int hh = 0; hh < n; ++hh) {
                        int h = hk * n + hh;
                        double s = 0.0;
                        for (int c = 0; c < D; ++c) {
                            double qc = oracle_widen(q[((size_t)b * H + h) * D + c], dtype);
                            double a = qc * oracle_widen(stats[base + c], dtype);
                            double m = qc * oracle_widen(stats[base + D + c], dtype);
                            s += a > m ? a : m;
                        }
                        if (logical_scores)
                            logical_scores[(((size_t)b * H + h) * max_pages + p) * g + j] = s;
                        if (!have || s > best) { best = s; have = 1; }
                    }
                }
                *dst = best;
            }
        }
    }
}

/* ---- top-K physical pages under the token budget (Sec. 3.5.2, Sec. 3.2) --------------- */
/*
 * K = budget_tokens / NP pages.  P = ceil(L / NP) pages exist.
 *   P <= K : every page is selected.
 *   else   : the page of the newest token (P-1) is taken first, then the K-1 pages of highest
 *            score among the rest, one at a time, a tie going to the lower page index.
 * The list is written ascending; sel_count = its length; sel_seq_len[b] = L.
 * sel_pages is [batch][Hkv][k_stride]; unused tail entries are set to -1.
 */
void oracle_select_pages(const double *page_scores, const int32_t *seq_lens, int batch, int Hkv,
                         int max_pages, int NP, int budget_tokens, int k_stride,
                         int32_t *sel_pages, int32_t *sel_count, int32_t *sel_seq_len)
{
    int K = budget_tokens / NP;
    for (int b = 0; b < batch; ++b) {
        int L = seq_lens[b];
        int P = ceil_div(L, NP);
        sel_seq_len[b] = L;
        for (int hk = 0; hk < Hkv; ++hk) {
            const double *sc = &page_scores[((size_t)b * Hkv + hk) * max_pages];
            int32_t *out = &sel_pages[((size_t)b * Hkv + hk) * k_stride];
            unsigned char *taken = (unsigned char *)calloc((size_t)(P > 0 ? P : 1), 1);
            int count = 0;
            if (P <= K) {
                for (int p = 0; p < P; ++p) taken[p] = 1;
                count = P;
            } else {
                taken[P - 1] = 1;
                count = 1;
                while (count < K) {
                    int arg = -1;
                    for (int p = 0; p < P; ++p) {
                        if (taken[p]) continue;
                        if (arg < 0 || sc[p] > sc[arg]) arg = p; /* strict: lower index wins ties */
                    }
                    taken[arg] = 1;
                    ++count;
                }
            }
            int w = 0;
            for (int p = 0; p < P; ++p)
                if (taken[p]) out[w++] = p;
            for (; w < k_stride; ++w) out[w] = -1;
            sel_count[(size_t)b * Hkv + hk] = count;
            free(taken);
        }
    }
}

/* ---- paged sparse decode (Eq. 1 over the pages of an index table; Sec. 3.6) ----------- */
/*
 * One query per sequence.  Page set of KV head hk at length L (P = ceil(L/NP) pages):
 *   streaming head: pages p < s  or  p > P-1-w,   s = ceil(sink/NP), w = ceil(local/NP);
 *   selecting head: the listed pages, plus every page p >= ceil(sel_seq_len/NP) (created after
 *                   the selection was made).
 * Attended tokens = tokens u < L of those pages.  For each query head h of the group:
 *   score_u = scale * q_h . k_u,  out_h = sum_u softmax(score)_u * v_u,  lse_h = log sum_u exp(score_u).
 */
/* Element of a KV pool: 16-bit storage, or (k64 / v64 given) a pool of doubles holding the values a
 * quantised cache stands for. */
static inline double pool_value(const uint16_t *p16, const double *p64, size_t idx, int dtype)
{
    return p64 ? p64[idx] : oracle_widen(p16[idx], dtype);
}

static void sparse_decode_any(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                              const double *k64, const double *v64,
                              const int32_t *page_table, const int32_t *seq_lens,
                              const int32_t *sel_pages, const int32_t *sel_count,
                              const int32_t *sel_seq_len, int k_stride,
                              const uint8_t *kv_head_is_streaming, int batch, int max_pages, int H,
                              int Hkv, int D, int NP, int dtype, int sink_tokens, int local_tokens,
                              double sm_scale, double *out, double *lse)
{
    int n = H / Hkv;
    int s = ceil_div(sink_tokens, NP);
    int w = ceil_div(local_tokens, NP);
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < batch * H; ++bh) {
        int b = bh / H, h = bh % H, hk = h / n;
        int L = seq_lens[b];
        int P = ceil_div(L, NP);
        unsigned char *use = (unsigned char *)calloc((size_t)P, 1);
        if (kv_head_is_streaming[hk]) {
            for (int p = 0; p < P; ++p)
                if (p < s || p > P - 1 - w) use[p] = 1;
        } else {
            int cnt = sel_count[(size_t)b * Hkv + hk];
            for (int i = 0; i < cnt; ++i) {
                int p = sel_pages[((size_t)b * Hkv + hk) * k_stride + i];
                if (p >= 0 && p < P) use[p] = 1;
            }
            for (int p = ceil_div(sel_seq_len[b], NP); p < P; ++p) use[p] = 1;
        }
        double *score = (double *)malloc(sizeof(double) * (size_t)P * NP);
        int *pos = (int *)malloc(sizeof(int) * (size_t)P * NP);
        int m = 0;
        const uint16_t *qh = &q[((size_t)b * H + h) * D];
        for (int p = 0; p < P; ++p) {
            if (!use[p]) continue;
            int page = page_table[(size_t)b * max_pages + p];
            for (int t = 0; t < NP && p * NP + t < L; ++t) {
                double dot = 0.0;
                for (int c = 0; c < D; ++c)
                    dot += oracle_widen(qh[c], dtype) *
                           pool_value(k_pool, k64, pool_index(page, hk, t, c, Hkv, NP, D), dtype);
                score[m] = dot * sm_scale;
                pos[m] = p * NP + t;
                ++m;
            }
        }
        double mx = -INFINITY;
        for (int i = 0; i < m; ++i) mx = score[i] > mx ? score[i] : mx;
        double denom = 0.0;
        for (int i = 0; i < m; ++i) denom += exp(score[i] - mx);
        double *o = &out[((size_t)b * H + h) * D];
        for (int c = 0; c < D; ++c) o[c] = 0.0;
        for (int i = 0; i < m; ++i) {
            double pr = exp(score[i] - mx) / denom;
            int page = page_table[(size_t)b * max_pages + pos[i] / NP];
            for (int c = 0; c < D; ++c)
                o[c] += pr * pool_value(v_pool, v64, pool_index(page, hk, pos[i] % NP, c, Hkv, NP, D), dtype);
        }
        if (lse) lse[(size_t)b * H + h] = mx + log(denom);
        free(use); free(score); free(pos);
    }
}

void oracle_sparse_decode(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                          const int32_t *page_table, const int32_t *seq_lens,
                          const int32_t *sel_pages, const int32_t *sel_count,
                          const int32_t *sel_seq_len, int k_stride,
                          const uint8_t *kv_head_is_streaming, int batch, int max_pages, int H,
                          int Hkv, int D, int NP, int dtype, int sink_tokens, int local_tokens,
                          double sm_scale, double *out, double *lse)
{
    sparse_decode_any(q, k_pool, v_pool, NULL, NULL, page_table, seq_lens, sel_pages, sel_count,
                      sel_seq_len, k_stride, kv_head_is_streaming, batch, max_pages, H, Hkv, D, NP,
                      dtype, sink_tokens, local_tokens, sm_scale, out, lse);
}

/* The same decode over a quantised cache (Sec. 3.2, Sec. 3.6): the pools hold, as doubles, the values
 * code * scale + zero that the stored bytes stand for; queries stay in 16-bit storage. */
void oracle_sparse_decode_values(const uint16_t *q, const double *k_values, const double *v_values,
                                 const int32_t *page_table, const int32_t *seq_lens,
                                 const int32_t *sel_pages, const int32_t *sel_count,
                                 const int32_t *sel_seq_len, int k_stride,
                                 const uint8_t *kv_head_is_streaming, int batch, int max_pages,
                                 int H, int Hkv, int D, int NP, int dtype, int sink_tokens,
                                 int local_tokens, double sm_scale, double *out, double *lse)
{
    sparse_decode_any(q, NULL, NULL, k_values, v_values, page_table, seq_lens, sel_pages, sel_count,
                      sel_seq_len, k_stride, kv_head_is_streaming, batch, max_pages, H, Hkv, D, NP,
                      dtype, sink_tokens, local_tokens, sm_scale, out, lse);
}

/* ---- block-sparse prefill, one (token, head) row at a time (Eq. 1 + Sec. 3.1 mask) ----- */
/*
 * Tokens of all sequences are concatenated; cu_seqlens[b] is the first token of sequence b.
 * Row r asks for global token rows_token[r] and query head rows_head[r].  With t the position
 * inside its sequence and T the tile size, key position u is allowed iff u <= t and
 *   dense head    : always;
 *   streaming head: tile(u) < s  or  tile(u) > tile(t) - w,  tile(x) = x / T,
 *                   s = ceil(sink/T), w = ceil(local/T).
 * out is [n_rows][D], lse [n_rows] (may be NULL).
 */
void oracle_sparse_prefill_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                                const int32_t *cu_seqlens, int batch, int H, int Hkv, int D,
                                int dtype, int T, int sink_tokens, int local_tokens,
                                const uint8_t *kv_head_is_streaming, double sm_scale,
                                const int32_t *rows_token, const int32_t *rows_head, int n_rows,
                                double *out, double *lse)
{
    int n = H / Hkv;
    int s = ceil_div(sink_tokens, T);
    int w = ceil_div(local_tokens, T);
#pragma omp parallel for schedule(dynamic, 4)
    for (int r = 0; r < n_rows; ++r) {
        int tok = rows_token[r], h = rows_head[r], hk = h / n;
        int b = 0;
        while (b + 1 < batch && cu_seqlens[b + 1] <= tok) ++b;
        int start = cu_seqlens[b];
        int t = tok - start;
        int streaming = kv_head_is_streaming[hk];
        double *score = (double *)malloc(sizeof(double) * (size_t)(t + 1));
        const uint16_t *qh = &q[((size_t)tok * H + h) * D];
        double mx = -INFINITY;
        for (int u = 0; u <= t; ++u) {
            int allowed = !streaming || (u / T < s) || (u / T > t / T - w);
            if (!allowed) { score[u] = -INFINITY; continue; }
            const uint16_t *ku = &k[((size_t)(start + u) * Hkv + hk) * D];
            double dot = 0.0;
            for (int c = 0; c < D; ++c)
                dot += oracle_widen(qh[c], dtype) * oracle_widen(ku[c], dtype);
            score[u] = dot * sm_scale;
            if (score[u] > mx) mx = score[u];
        }
        double denom = 0.0;
        for (int u = 0; u <= t; ++u)
            if (score[u] != -INFINITY) denom += exp(score[u] - mx);
        double *o = &out[(size_t)r * D];
        for (int c = 0; c < D; ++c) o[c] = 0.0;
        for (int u = 0; u <= t; ++u) {
            if (score[u] == -INFINITY) continue;
            double pr = exp(score[u] - mx) / denom;
            const uint16_t *vu = &v[((size_t)(start + u) * Hkv + hk) * D];
            for (int c = 0; c < D; ++c) o[c] += pr * oracle_widen(vu[c], dtype);
        }
        if (lse) lse[r] = mx + log(denom);
        free(score);
    }
}

/* ---- chunked prefill over a paged cache (Sec. 2.1: prefill with S tokens of KV history; Sec. 3.1 mask) ---- */
/*
 * The K / V of every token, the chunk's own included, sit in the paged pools; sequence b has L_b =
 * seq_lens[b] tokens and its chunk holds the last n_b = cu_q[b+1] - cu_q[b] of them, so query j of the
 * chunk is the token at position t = L_b - n_b + j.  It attends the positions u <= t allowed by the same
 * tile-granular mask as oracle_sparse_prefill_rows, with tiles counted from position 0 of the sequence.
 * Row r asks for chunk token rows_token[r] (index into q) and query head rows_head[r].
 */
void oracle_paged_prefill_rows(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                               const int32_t *page_table, const int32_t *seq_lens, const int32_t *cu_q,
                               int batch, int max_pages, int H, int Hkv, int D, int NP, int dtype,
                               int sink_tokens, int local_tokens, const uint8_t *kv_head_is_streaming,
                               double sm_scale, const int32_t *rows_token, const int32_t *rows_head,
                               int n_rows, double *out, double *lse)
{
    int n = H / Hkv;
    int s = ceil_div(sink_tokens, NP);
    int w = ceil_div(local_tokens, NP);
#pragma omp parallel for schedule(dynamic, 4)
    for (int r = 0; r < n_rows; ++r) {
        int tok = rows_token[r], h = rows_head[r], hk = h / n;
        int b = 0;
        while (b + 1 < batch && cu_q[b + 1] <= tok) ++b;
        int t = seq_lens[b] - (cu_q[b + 1] - cu_q[b]) + (tok - cu_q[b]);
        int streaming = kv_head_is_streaming[hk];
        double *score = (double *)malloc(sizeof(double) * (size_t)(t + 1));
        const uint16_t *qh = &q[((size_t)tok * H + h) * D];
        double mx = -INFINITY;
        for (int u = 0; u <= t; ++u) {
            int allowed = !streaming || (u / NP < s) || (u / NP > t / NP - w);
            if (!allowed) { score[u] = -INFINITY; continue; }
            int page = page_table[(size_t)b * max_pages + u / NP];
            double dot = 0.0;
            for (int c = 0; c < D; ++c)
                dot += oracle_widen(qh[c], dtype) *
                       oracle_widen(k_pool[pool_index(page, hk, u % NP, c, Hkv, NP, D)], dtype);
            score[u] = dot * sm_scale;
            if (score[u] > mx) mx = score[u];
        }
        double denom = 0.0;
        for (int u = 0; u <= t; ++u)
            if (score[u] != -INFINITY) denom += exp(score[u] - mx);
        double *o = &out[(size_t)r * D];
        for (int c = 0; c < D; ++c) o[c] = 0.0;
        for (int u = 0; u <= t; ++u) {
            if (score[u] == -INFINITY) continue;
            double pr = exp(score[u] - mx) / denom;
            int page = page_table[(size_t)b * max_pages + u / NP];
            for (int c = 0; c < D; ++c)
                o[c] += pr * oracle_widen(v_pool[pool_index(page, hk, u % NP, c, Hkv, NP, D)], dtype);
        }
        if (lse) lse[r] = mx + log(denom);
        free(score);
    }
}

/* ---- chunked prefill in the order of the prefill flow (Sec. 3.2: attention first, write-back after; Sec. 2.1:
 *      N new tokens with S tokens of history) ---------------------------------------------------------------- */
/*
 * Sequence b has hist_lens[b] = S_b tokens in its cache and n_b = cu_new[b+1] - cu_new[b] new tokens whose Q, K, V
 * arrive contiguously; query j of the chunk sits at position t = S_b + j.  It attends the positions u <= t allowed
 * by the tile-granular mask of oracle_sparse_prefill_rows (tiles counted from position 0): a history token u < S_b
 * with the key / value the cache stands for, given as doubles in k_hist / v_hist [batch][hist_stride][Hkv][D]
 * (gathered, and for a quantised cache dequantised, by the caller; a position the cache no longer holds may be NaN
 * there: a streaming head must never touch it), a chunk token u >= S_b with k_new / v_new [total_new][Hkv][D].
 * Row r asks for chunk token rows_token[r] (index into q) and query head rows_head[r].
 */
void oracle_chunk_prefill_rows(const uint16_t *q, const uint16_t *k_new, const uint16_t *v_new,
                               const double *k_hist, const double *v_hist, const int32_t *hist_lens,
                               const int32_t *cu_new, int batch, int hist_stride, int H, int Hkv, int D,
                               int T, int dtype, int sink_tokens, int local_tokens,
                               const uint8_t *kv_head_is_streaming, double sm_scale,
                               const int32_t *rows_token, const int32_t *rows_head, int n_rows, double *out,
                               double *lse)
{
    int n = H / Hkv;
    int s = ceil_div(sink_tokens, T);
    int w = ceil_div(local_tokens, T);
#pragma omp parallel for schedule(dynamic, 4)
    for (int r = 0; r < n_rows; ++r) {
        int tok = rows_token[r], h = rows_head[r], hk = h / n;
        int b = 0;
        while (b + 1 < batch && cu_new[b + 1] <= tok) ++b;
        int S = hist_lens[b];
        int t = S + (tok - cu_new[b]);
        int streaming = kv_head_is_streaming[hk];
        double *score = (double *)malloc(sizeof(double) * (size_t)(t + 1));
        const uint16_t *qh = &q[((size_t)tok * H + h) * D];
        double mx = -INFINITY;
        for (int u = 0; u <= t; ++u) {
            int allowed = !streaming || (u / T < s) || (u / T > t / T - w);
            if (!allowed) { score[u] = -INFINITY; continue; }
            double dot = 0.0;
            for (int c = 0; c < D; ++c) {
                double kc = u < S ? k_hist[(((size_t)b * hist_stride + u) * Hkv + hk) * D + c]
                                  : oracle_widen(k_new[((size_t)(cu_new[b] + u - S) * Hkv + hk) * D + c], dtype);
                dot += oracle_widen(qh[c], dtype) * kc;
            }
            score[u] = dot * sm_scale;
            if (score[u] > mx) mx = score[u];
        }
        double denom = 0.0;
        for (int u = 0; u <= t; ++u)
            if (score[u] != -INFINITY) denom += exp(score[u] - mx);
        double *o = &out[(size_t)r * D];
        for (int c = 0; c < D; ++c) o[c] = 0.0;
        for (int u = 0; u <= t; ++u) {
            if (score[u] == -INFINITY) continue;
            double pr = exp(score[u] - mx) / denom;
            for (int c = 0; c < D; ++c) {
                double vc = u < S ? v_hist[(((size_t)b * hist_stride + u) * Hkv + hk) * D + c]
                                  : oracle_widen(v_new[((size_t)(cu_new[b] + u - S) * Hkv + hk) * D + c], dtype);
                o[c] += pr * vc;
            }
        }
        if (lse) lse[r] = mx + log(denom);
        free(score);
    }
}

/* ---- prefill under a general block mask (Sec. 3.1: every tile is skipped or computed whole; Sec. 3.4:
 *      the kernel walks whatever list of key tiles it is given) --------------------------------------- */
/*
 * As oracle_sparse_prefill_rows, but the kept tiles of query head h come from a list: head_mask[h] = m >= 0
 * names mask m, whose row for query tile i of sequence b is cols[row_ptr[r] .. row_ptr[r + 1]) with
 * r = m * rows_per_mask + q_tile_start[b] + i; key position u is allowed iff u <= t and tile(u) is listed in
 * the row of tile(t).  head_mask[h] = -1 keeps the analytic mask (dense or streaming) of the other function.
 * A row with no allowed key gives out = 0 and lse = -inf.
 */
void oracle_block_mask_prefill_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                                    const int32_t *cu_seqlens, int batch, int H, int Hkv, int D, int dtype,
                                    int T, int sink_tokens, int local_tokens,
                                    const uint8_t *kv_head_is_streaming, double sm_scale,
                                    const int32_t *head_mask, const int32_t *q_tile_start,
                                    const int32_t *row_ptr, const int32_t *cols, int rows_per_mask,
                                    const int32_t *rows_token, const int32_t *rows_head, int n_rows,
                                    double *out, double *lse)
{
    int n = H / Hkv;
    int s = ceil_div(sink_tokens, T);
    int w = ceil_div(local_tokens, T);
#pragma omp parallel for schedule(dynamic, 4)
    for (int r = 0; r < n_rows; ++r) {
        int tok = rows_token[r], h = rows_head[r], hk = h / n;
        int b = 0;
        while (b + 1 < batch && cu_seqlens[b + 1] <= tok) ++b;
        int start = cu_seqlens[b];
        int t = tok - start;
        int m = head_mask[h];
        int lo = 0, hi = 0;
        if (m >= 0) {
            int row = m * rows_per_mask + q_tile_start[b] + t / T;
            lo = row_ptr[row];
            hi = row_ptr[row + 1];
        }
        double *score = (double *)malloc(sizeof(double) * (size_t)(t + 1));
        const uint16_t *qh = &q[((size_t)tok * H + h) * D];
        double mx = -INFINITY;
        for (int u = 0; u <= t; ++u) {
            int allowed;
            if (m >= 0) {
                allowed = 0;
                for (int e = lo; e < hi; ++e)
                    if (cols[e] == u / T) allowed = 1;
            } else {
                allowed = !kv_head_is_streaming[hk] || (u / T < s) || (u / T > t / T - w);
            }
            if (!allowed) { score[u] = -INFINITY; continue; }
            const uint16_t *ku = &k[((size_t)(start + u) * Hkv + hk) * D];
            double dot = 0.0;
            for (int c = 0; c < D; ++c)
                dot += oracle_widen(qh[c], dtype) * oracle_widen(ku[c], dtype);
            score[u] = dot * sm_scale;
            if (score[u] > mx) mx = score[u];
        }
        double denom = 0.0;
        for (int u = 0; u <= t; ++u)
            if (score[u] != -INFINITY) denom += exp(score[u] - mx);
        double *o = &out[(size_t)r * D];
        for (int c = 0; c < D; ++c) o[c] = 0.0;
        if (denom > 0.0) {
            for (int u = 0; u <= t; ++u) {
                if (score[u] == -INFINITY) continue;
                double pr = exp(score[u] - mx) / denom;
                const uint16_t *vu = &v[((size_t)(start + u) * Hkv + hk) * D];
                for (int c = 0; c < D; ++c) o[c] += pr * oracle_widen(vu[c], dtype);
            }
        }
        if (lse) lse[r] = denom > 0.0 ? mx + log(denom) : -INFINITY;
        free(score);
    }
}

/* ---- block counting (Sec. 3.1: cost ~ number of non-empty tiles, speed-up 1/(1-r)) ---- */
/*
 * Number of T x T tiles of an n_tokens causal prefill that hold at least one allowed
 * (query, key) pair, by enumeration of every tile pair and every element inside it.
 */
long long oracle_count_nonempty_tiles(int n_tokens, int T, int sink_tokens, int local_tokens,
                                      int streaming)
{
    int s = ceil_div(sink_tokens, T);
    int w = ceil_div(local_tokens, T);
    int nt = ceil_div(n_tokens, T);
    long long count = 0;
    for (int i = 0; i < nt; ++i) {
        for (int j = 0; j < nt; ++j) {
            int any = 0;
            for (int t = i * T; t < (i + 1) * T && t < n_tokens && !any; ++t)
                for (int u = j * T; u < (j + 1) * T && u < n_tokens; ++u) {
                    int allowed = u <= t && (!streaming || (u / T < s) || (u / T > t / T - w));
                    if (allowed) { any = 1; break; }
                }
            count += any;
        }
    }
    return count;
}

/* Theoretical speed-up of block sparsity with r = (total - nonempty) / total: 1 / (1 - r). */
double oracle_block_sparse_speedup(long long nonempty_tiles, long long total_tiles)
{
    double r = (double)(total_tiles - nonempty_tiles) / (double)total_tiles;
    return 1.0 / (1.0 - r);
}
