// Hierarchical page selector (Sec. 3.5.2): Eq. 2 scores from the per-logical-page key statistics,
// max over the query heads of a GQA group and over the logical pages of a physical page, then the
// top-K physical pages per (sequence, KV head).
//
// Scoring is a bandwidth-bound scan of the statistics (2 KiB per page and head for N_P = 64,
// N_L = 16): 16 lanes read the max row and the min row of one logical page with 16-byte loads.
// Because kmax >= kmin, max(q*kmax, q*kmin) = max(q,0)*kmax + min(q,0)*kmin, so each channel costs
// two packed dot-product lanes and no compare.  Top-K ranks an order-preserving integer image of the
// fp32 score: lists of up to 8192 candidates from registers, on ballots alone; longer ones from memory
// with a 4-pass radix select.  Both emit in index order, so the output is ascending and ties resolve
// to the lower page index.
#include "kernels.h"

namespace lserve {

namespace {

constexpr int kScoreThreads = 256;  // 4 waves, 4 pages per wave (one per 16-lane row)
constexpr int kPagesPerBlock = 16;
constexpr int kTopkThreads = 512;
constexpr int kTopkLdsKeys = 8192;  // up to 8192 candidate pages (524288 tokens at N_P = 64) are ranked from LDS

__device__ __forceinline__ unsigned orderable(float s) {
    unsigned u = __builtin_bit_cast(unsigned, s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// GMAX: upper bound of the logical pages per physical page (4 or kMaxLogical), sizes the row registers.
template <class T, int N, int GMAX>
__global__ __launch_bounds__(kScoreThreads) void page_score_kernel(LayerParams lp, PagedParams kv,
                                                                    const uint4* __restrict__ q,
                                                                    const int* __restrict__ stats_valid_len,
                                                                    float* __restrict__ scores, HeadList heads) {
    const int b = blockIdx.z;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int r = lane / 16, c = lane % 16;
    const int L = kv.seq_lens[b];
    const int P = ceil_div(L, lp.NP);
    // (page, selecting head) pairs with the head running fastest: the statistics of the heads of one page
    // are neighbours in memory, so the rows of a wave read one contiguous stretch
    const int pair = (blockIdx.x * (kScoreThreads / kWave) + wave) * 4 + r;
    const int p = pair / heads.count;
    if (p >= kv.max_pages) return;
    const int hk = heads.idx[pair % heads.count];
    float* dst = scores + ((size_t)b * lp.Hkv + hk) * kv.max_pages + p;
    // Pages past the end of the sequence have no score: nothing reads one (the ranking stops at the last page),
    // and a caller's score array gets its zeros there from the ranking kernel, in whole lines.  Written from
    // here, one 4-byte store per (page, head) into lists max_pages apart, the zeros of a ragged batch cost more
    // than its scores: 124 -> 107 us per selector run on 32 sequences of 4K .. 128K tokens.
    if (p >= P) return;  // whole row (16 lanes) takes this branch together

    // positive and negative parts of the group's queries for this lane's 8 channels
    uint32_t qpos[N][4], qneg[N][4];
#pragma unroll
    for (int hh = 0; hh < N; ++hh) {
        uint4 x = q[((size_t)b * lp.H + hk * N + hh) * (kHeadDim / 8) + c];
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float a = Elem<T>::lo(w[i]), d = Elem<T>::hi(w[i]);
            qpos[hh][i] = Elem<T>::pack(fmaxf(a, 0.f), fmaxf(d, 0.f));
            qneg[hh][i] = Elem<T>::pack(fminf(a, 0.f), fminf(d, 0.f));
        }
    }

    const int phys = kv.page_table[(size_t)b * kv.max_pages + p];
    const size_t ph = (size_t)phys * kv.pool_heads + pool_rank(lp, kv, hk, false);  // (page, head) index inside the main pool
    uint4* st = reinterpret_cast<uint4*>(kv.stats) + ph * lp.g * 2 * (kHeadDim / 8);
    const int fresh_below = stats_valid_len ? stats_valid_len[b] : L;  // stored statistics cover tokens below this
    // Rows of every logical page with a valid token.  All stored rows are requested before any is used, so a
    // wavefront has its whole 2 KiB per pair in flight at once: with one logical page at a time the loads in
    // flight per compute unit capped the scan near half the memory bandwidth.  Logical pages that received
    // tokens since the statistics were last brought up to date (at most the tail of the sequence) are rebuilt
    // from their keys afterwards (lane c owns channels 8c .. 8c+7), used and stored.
    const int n_log = min(lp.g, ceil_div(L - p * lp.NP, lp.NL));
    uint4 mx[GMAX], mn[GMAX];
    bool any_stale = false;
#pragma unroll
    for (int j = 0; j < GMAX; ++j) {
        if (j < n_log) {
            const int lo = p * lp.NP + j * lp.NL;
            if (min(lo + lp.NL, L) > fresh_below) {
                any_stale = true;
            } else {
                mx[j] = st[(size_t)(j * 2) * (kHeadDim / 8) + c];
                mn[j] = st[(size_t)(j * 2 + 1) * (kHeadDim / 8) + c];
            }
        }
    }
    if (any_stale) {
#pragma unroll
        for (int j = 0; j < GMAX; ++j) {
            const int lo = p * lp.NP + j * lp.NL;
            if (j < n_log && min(lo + lp.NL, L) > fresh_below) {
                const uint4* keys = reinterpret_cast<const uint4*>(kv.k_pool) +
                                    (ph * lp.NP + (lo - p * lp.NP)) * (kHeadDim / 8) + c;
                float vmax[8], vmin[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    vmax[i] = -INFINITY;
                    vmin[i] = INFINITY;
                }
                const int cnt = min(lp.NL, L - lo);
                for (int t0 = 0; t0 < cnt; t0 += 8) {  // eight rows requested together
                    uint4 x[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        x[u] = keys[(size_t)min(t0 + u, cnt - 1) * (kHeadDim / 8)];  // a repeated row changes nothing
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const uint32_t w[4] = {x[u].x, x[u].y, x[u].z, x[u].w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float a = Elem<T>::lo(w[i]), d = Elem<T>::hi(w[i]);
                            vmax[2 * i] = fmaxf(vmax[2 * i], a);
                            vmin[2 * i] = fminf(vmin[2 * i], a);
                            vmax[2 * i + 1] = fmaxf(vmax[2 * i + 1], d);
                            vmin[2 * i + 1] = fminf(vmin[2 * i + 1], d);
                        }
                    }
                }
                mx[j] = make_uint4(Elem<T>::pack(vmax[0], vmax[1]), Elem<T>::pack(vmax[2], vmax[3]),
                                   Elem<T>::pack(vmax[4], vmax[5]), Elem<T>::pack(vmax[6], vmax[7]));
                mn[j] = make_uint4(Elem<T>::pack(vmin[0], vmin[1]), Elem<T>::pack(vmin[2], vmin[3]),
                                   Elem<T>::pack(vmin[4], vmin[5]), Elem<T>::pack(vmin[6], vmin[7]));
                st[(size_t)(j * 2) * (kHeadDim / 8) + c] = mx[j];
                st[(size_t)(j * 2 + 1) * (kHeadDim / 8) + c] = mn[j];
            }
        }
    }
    float best = -INFINITY;
#pragma unroll
    for (int j = 0; j < GMAX; ++j) {
        if (j < n_log) {
            const uint32_t wx[4] = {mx[j].x, mx[j].y, mx[j].z, mx[j].w};
            const uint32_t wn[4] = {mn[j].x, mn[j].y, mn[j].z, mn[j].w};
#pragma unroll
            for (int hh = 0; hh < N; ++hh) {
                float s = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) s = Elem<T>::dot2(qpos[hh][i], wx[i], s);
#pragma unroll
                for (int i = 0; i < 4; ++i) s = Elem<T>::dot2(qneg[hh][i], wn[i], s);
                best = fmaxf(best, row16_sum(s));
            }
        }
    }
    if (c == 0) *dst = best + 0.f;  // +0 canonicalises a negative zero
}

// Inclusive scan of (a, b) pairs over the block; returns this thread's exclusive prefix and the totals.
__device__ __forceinline__ void block_exclusive_scan2(int a, int b, int* lds /* 2 * waves */, int& ea, int& eb,
                                                      int& ta, int& tb) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave, nw = blockDim.x / kWave;
    int ia = a, ib = b;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int ua = __shfl_up(ia, d, kWave), ub = __shfl_up(ib, d, kWave);
        if (lane >= d) {
            ia += ua;
            ib += ub;
        }
    }
    if (lane == kWave - 1) {
        lds[wave] = ia;
        lds[nw + wave] = ib;
    }
    __syncthreads();
    int oa = 0, ob = 0;
    ta = 0;
    tb = 0;
    for (int w = 0; w < nw; ++w) {
        if (w < wave) {
            oa += lds[w];
            ob += lds[nw + w];
        }
        ta += lds[w];
        tb += lds[nw + w];
    }
    ea = oa + ia - a;
    eb = ob + ib - b;
    __syncthreads();
}

__global__ __launch_bounds__(kTopkThreads) void topk_pages_kernel(LayerParams lp, PagedParams kv, int K,
                                                                   const float* __restrict__ scores,
                                                                   float* __restrict__ user_scores,
                                                                   int* __restrict__ sel_pages,
                                                                   int* __restrict__ sel_count,
                                                                   int* __restrict__ sel_seq_len) {
    __shared__ int hist[256];
    __shared__ unsigned skeys[kTopkLdsKeys];  // the list's keys, when they fit: every pass then stays in LDS
    __shared__ int scan_lds[2 * kTopkThreads / kWave];
    __shared__ unsigned s_prefix;
    __shared__ int s_need;

    const int b = blockIdx.y, hk = blockIdx.x, tid = threadIdx.x;
    const int L = kv.seq_lens[b];
    const int P = ceil_div(L, lp.NP);
    int* out = sel_pages + ((size_t)b * lp.Hkv + hk) * K;
    if (hk == 0 && tid == 0) sel_seq_len[b] = L;

    if ((lp.streaming_mask >> hk) & 1ull) {  // streaming heads take no selection
        for (int i = tid; i < K; i += blockDim.x) out[i] = -1;
        if (user_scores)
            for (int i = tid; i < kv.max_pages; i += blockDim.x)
                user_scores[((size_t)b * lp.Hkv + hk) * kv.max_pages + i] = 0.f;
        if (tid == 0) sel_count[b * lp.Hkv + hk] = 0;
        return;
    }
    if (user_scores)  // a caller's array reads 0 past the sequence's last page
        for (int i = P + tid; i < kv.max_pages; i += blockDim.x)
            user_scores[((size_t)b * lp.Hkv + hk) * kv.max_pages + i] = 0.f;
    if (P <= K) {  // the budget covers the whole context
        for (int i = tid; i < K; i += blockDim.x) out[i] = i < P ? i : -1;
        if (tid == 0) sel_count[b * lp.Hkv + hk] = P;
        return;
    }

    const float* sc = scores + ((size_t)b * lp.Hkv + hk) * kv.max_pages;
    const int M = P - 1;  // candidates: every page but the newest, which is always kept
    const bool in_lds = M <= kTopkLdsKeys;
    if (in_lds) {
        for (int i = tid; i < M; i += blockDim.x) skeys[i] = orderable(sc[i]);
        __syncthreads();
    }
    auto key_at = [&](int i) { return in_lds ? skeys[i] : orderable(sc[i]); };
    int need = K - 1;     // how many candidates to take
    unsigned threshold = 0xffffffffu;
    int need_eq = 0;
    if (need > 0) {
        // radix select: after the four passes s_prefix is the key of the need-th best candidate
        if (tid == 0) {
            s_prefix = 0;
            s_need = need;
        }
        unsigned mask = 0;
        for (int shift = 24; shift >= 0; shift -= 8) {
            for (int i = tid; i < 256; i += blockDim.x) hist[i] = 0;
            __syncthreads();
            const unsigned prefix = s_prefix;
            for (int i = tid; i < M; i += blockDim.x) {
                unsigned key = key_at(i);
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
            }
            __syncthreads();
            if (tid < kWave) {
                // lane l owns buckets 255-4l .. 252-4l; walk from the highest bucket down
                int h0 = hist[255 - 4 * tid], h1 = hist[254 - 4 * tid], h2 = hist[253 - 4 * tid], h3 = hist[252 - 4 * tid];
                int tot = h0 + h1 + h2 + h3, inc = tot;
#pragma unroll
                for (int d = 1; d < kWave; d <<= 1) {
                    int u = __shfl_up(inc, d, kWave);
                    if (tid >= d) inc += u;
                }
                const int want = s_need;
                const int above = inc - tot;  // candidates in higher buckets than this lane's
                if (above < want && inc >= want) {
                    int bucket = 255 - 4 * tid, acc = above;
                    if (acc + h0 < want) {
                        acc += h0;
                        --bucket;
                        if (acc + h1 < want) {
                            acc += h1;
                            --bucket;
                            if (acc + h2 < want) {
                                acc += h2;
                                --bucket;
                            }
                        }
                    }
                    s_prefix = prefix | ((unsigned)bucket << shift);
                    s_need = want - acc;
                }
            }
            mask |= 0xffu << shift;
            __syncthreads();
        }
        threshold = s_prefix;
        need_eq = s_need;  // candidates equal to the threshold still to take, lowest indices first
    }

    // index-ordered compaction: each thread owns a contiguous range of pages
    const int per = ceil_div(M, (int)blockDim.x);
    const int i0 = min(M, tid * per), i1 = min(M, i0 + per);
    int gt = 0, eq = 0;
    for (int i = i0; i < i1; ++i) {
        unsigned key = key_at(i);
        gt += key > threshold;
        eq += key == threshold;
    }
    int egt, eeq, tgt, teq;
    block_exclusive_scan2(gt, eq, scan_lds, egt, eeq, tgt, teq);
    int pos = egt + min(eeq, need_eq);
    int eq_seen = eeq;
    for (int i = i0; i < i1; ++i) {
        unsigned key = key_at(i);
        bool take = key > threshold;
        if (key == threshold) {
            take = eq_seen < need_eq;
            ++eq_seen;
        }
        if (take && pos < K - 1) out[pos++] = i;  // the bound only matters for non-finite scores
    }
    if (tid == 0) {
        out[K - 1] = P - 1;
        sel_count[b * lp.Hkv + hk] = K;
    }
}

// The same selection on ballots alone, for lists of up to 64 * KPL * WAVES candidate pages: WAVES wavefronts share
// a list, each keeping the keys of 64 * KPL consecutive pages in registers (lane l holds pages l, l + 64, ... of
// its wavefront's stretch).  The key of the (K - 1)-th best candidate is found bit by bit from the top (the largest
// t with at least K - 1 keys >= t): a step is one compare and one ballot per register and, with more than one
// wavefront, one barrier to add up their counts.  Nothing is histogrammed, so keys that agree in their leading
// bytes (page scores do: same sign, neighbouring exponents) cost nothing extra, where shared-memory atomics on a
// few hot buckets serialise.  Candidates above the threshold are taken, those equal to it in index order until the
// budget is full; a ballot per row of 64 pages places every taken page, so the output is ascending.
template <int KPL, int WAVES>
__global__ __launch_bounds__(kWave* WAVES) void topk_pages_ballot_kernel(LayerParams lp, PagedParams kv, int K,
                                                                         const float* __restrict__ scores,
                                                                         float* __restrict__ user_scores,
                                                                         int* __restrict__ sel_pages,
                                                                         int* __restrict__ sel_count,
                                                                         int* __restrict__ sel_seq_len) {
    __shared__ int counts[2][WAVES];     // per-wavefront counts of a search step, double buffered
    __shared__ int above_eq[2][WAVES];   // per-wavefront candidates above / equal to the threshold
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave, tid = threadIdx.x;
    const int list = blockIdx.x;
    const int b = list / lp.Hkv, hk = list % lp.Hkv;
    const int L = kv.seq_lens[b];
    const int P = ceil_div(L, lp.NP);
    int* out = sel_pages + (size_t)list * K;
    if (hk == 0 && tid == 0) sel_seq_len[b] = L;

    if ((lp.streaming_mask >> hk) & 1ull) {  // streaming heads take no selection
        for (int i = tid; i < K; i += kWave * WAVES) out[i] = -1;
        if (user_scores)
            for (int i = tid; i < kv.max_pages; i += kWave * WAVES) user_scores[(size_t)list * kv.max_pages + i] = 0.f;
        if (tid == 0) sel_count[list] = 0;
        return;
    }
    if (P <= K) {  // the budget covers the whole context
        for (int i = tid; i < K; i += kWave * WAVES) out[i] = i < P ? i : -1;
        if (tid == 0) sel_count[list] = P;
        if (user_scores)  // a caller's array reads 0 past the sequence's last page
            for (int i = P + tid; i < kv.max_pages; i += kWave * WAVES) user_scores[(size_t)list * kv.max_pages + i] = 0.f;
        return;
    }

    const float* sc = scores + (size_t)list * kv.max_pages;
    const int M = P - 1;  // candidates: every page but the newest, which is always kept
    const int first = wave * (KPL * kWave) + lane;  // this lane's pages: first, first + 64, ...
    // All loads first and without conditions (a guarded load is a branch, and the loads would then be waited for
    // one by one); rows past the end read the last candidate again and are blanked afterwards.
    float raw[KPL];
#pragma unroll
    for (int j = 0; j < KPL; ++j) raw[j] = sc[min(first + kWave * j, M - 1)];
    unsigned key[KPL];  // 0 stands for "no page": below the key of every number
#pragma unroll
    for (int j = 0; j < KPL; ++j) key[j] = first + kWave * j < M ? orderable(raw[j]) : 0u;

    // sum over the wavefronts of the list of a count every lane of a wavefront agrees on
    auto all_waves = [&](int mine, int (*slots)[WAVES], int phase) {
        if (WAVES == 1) return mine;
        if (lane == 0) slots[phase & 1][wave] = mine;
        __syncthreads();
        int total = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) total += slots[phase & 1][w];
        return total;
    };

    const int need = K - 1;
    unsigned threshold = 0xffffffffu;
    int need_eq = 0;
    if (need > 0) {
        unsigned prefix = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const unsigned t = prefix | (1u << bit);
            int at_least = 0;
#pragma unroll
            for (int j = 0; j < KPL; ++j) at_least += __popcll(__ballot(key[j] >= t));
            if (all_waves(at_least, counts, bit) >= need) prefix = t;
        }
        threshold = prefix;
    }
    int above = 0, equal = 0;
#pragma unroll
    for (int j = 0; j < KPL; ++j) {
        above += __popcll(__ballot(key[j] > threshold));
        equal += __popcll(__ballot(first + kWave * j < M && key[j] == threshold));
    }
    // candidates of the wavefronts before this one: those above the threshold, and those equal to it
    int above_before = 0, equal_before = 0, above_all = above;
    if (WAVES > 1) {
        if (lane == 0) {
            above_eq[0][wave] = above;
            above_eq[1][wave] = equal;
        }
        __syncthreads();
        above_all = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            above_all += above_eq[0][w];
            if (w < wave) {
                above_before += above_eq[0][w];
                equal_before += above_eq[1][w];
            }
        }
    }
    if (need > 0) need_eq = need - above_all;  // candidates equal to the threshold still to take, lowest indices first
    const unsigned long long lower_lanes = (1ull << lane) - 1ull;
    int taken = above_before + min(equal_before, need_eq), eq_seen = equal_before;
#pragma unroll
    for (int j = 0; j < KPL; ++j) {
        const int i = first + kWave * j;
        const bool is_eq = i < M && key[j] == threshold;
        const unsigned long long eq_row = __ballot(is_eq);
        const bool take = i < M && (key[j] > threshold || (is_eq && eq_seen + __popcll(eq_row & lower_lanes) < need_eq));
        const unsigned long long take_row = __ballot(take);
        const int pos = taken + __popcll(take_row & lower_lanes);
        if (take && pos < K - 1) out[pos] = i;  // the bound only matters for non-finite scores
        taken += __popcll(take_row);
        eq_seen += __popcll(eq_row);
    }
    if (tid == 0) {
        out[K - 1] = P - 1;
        sel_count[list] = K;
    }
    // a caller's array reads 0 past the sequence's last page (last, so that it costs the search no registers)
    if (user_scores)
        for (int i = P + tid; i < kv.max_pages; i += kWave * WAVES) user_scores[(size_t)list * kv.max_pages + i] = 0.f;
}

template <class T>
hipError_t launch_score(const LayerParams& lp, const PagedParams& kv, const void* q, const int* stats_valid_len,
                        float* scores, const HeadList& selecting, hipStream_t stream) {
    dim3 grid(ceil_div(kv.max_pages * selecting.count, kPagesPerBlock), 1, kv.batch);
    dim3 block(kScoreThreads);
    const uint4* q4 = reinterpret_cast<const uint4*>(q);
#define LSERVE_SCORE_CASE(N)                                                                                   \
    case N:                                                                                                    \
        if (lp.g <= 4)                                                                                         \
            hipLaunchKernelGGL((page_score_kernel<T, N, 4>), grid, block, 0, stream, lp, kv, q4, stats_valid_len,  \
                               scores, selecting);                                                             \
        else                                                                                                   \
            hipLaunchKernelGGL((page_score_kernel<T, N, kMaxLogical>), grid, block, 0, stream, lp, kv, q4,         \
                               stats_valid_len, scores, selecting);                                            \
        break;
    switch (lp.group) {
        LSERVE_SCORE_CASE(1)
        LSERVE_SCORE_CASE(2)
        LSERVE_SCORE_CASE(3)
        LSERVE_SCORE_CASE(4)
        LSERVE_SCORE_CASE(5)
        LSERVE_SCORE_CASE(6)
        LSERVE_SCORE_CASE(7)
        LSERVE_SCORE_CASE(8)
        default:
            return hipErrorInvalidValue;
    }
#undef LSERVE_SCORE_CASE
    return hipGetLastError();
}

}  // namespace

hipError_t preload_select_kernels() {
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&topk_pages_kernel));
}

hipError_t launch_select_pages(int dtype, const LayerParams& lp, const PagedParams& kv, const void* q,
                               const int* stats_valid_len, int budget_pages, int* sel_pages, int* sel_count, int* sel_seq_len,
                               float* scores, bool scores_is_user_buffer, const HeadList& selecting,
                               hipStream_t stream) {
    if (selecting.count > 0) {
        hipError_t e = dtype == 0 ? launch_score<F16>(lp, kv, q, stats_valid_len, scores, selecting, stream)
                                  : launch_score<BF16>(lp, kv, q, stats_valid_len, scores, selecting, stream);
        if (e != hipSuccess) return e;
    }
    float* user_scores = scores_is_user_buffer ? scores : nullptr;
    const int candidates = kv.max_pages - 1;  // no list has more
#define LSERVE_TOPK_BALLOT(KPL, WAVES)                                                                                  \
    hipLaunchKernelGGL((topk_pages_ballot_kernel<KPL, WAVES>), dim3(kv.batch * lp.Hkv), dim3(kWave * WAVES), 0, stream, \
                       lp, kv, budget_pages, scores, user_scores, sel_pages, sel_count, sel_seq_len)
    if (candidates <= kWave * 4) {
        LSERVE_TOPK_BALLOT(4, 1);
    } else if (candidates <= kWave * 8) {
        LSERVE_TOPK_BALLOT(8, 1);
    } else if (candidates <= kWave * 8 * 4) {
        LSERVE_TOPK_BALLOT(8, 4);
    } else if (candidates <= kWave * 8 * 8) {
        LSERVE_TOPK_BALLOT(8, 8);
    } else if (candidates <= kWave * 16 * 8) {
        LSERVE_TOPK_BALLOT(16, 8);
    } else {  // beyond 8192 candidate pages the keys stay in memory
        hipLaunchKernelGGL(topk_pages_kernel, dim3(lp.Hkv, kv.batch), dim3(kTopkThreads), 0, stream, lp, kv, budget_pages,
                           scores, user_scores, sel_pages, sel_count, sel_seq_len);
    }
#undef LSERVE_TOPK_BALLOT
    return hipGetLastError();
}

}  // namespace lserve
