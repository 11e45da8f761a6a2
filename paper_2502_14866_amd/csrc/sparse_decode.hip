// Paged sparse decode attention (Sec. 3.6): one query token per sequence attends only the pages of
// its index table -- the selector's list (plus pages newer than the selection) for dense heads,
// sink + local pages for streaming heads.  Both kinds run in one launch.
//
// The work is GEMV-shaped (n <= 8 query rows per KV head) and bound by HBM bandwidth, so there is
// no MFMA here: each page is a 2 * N_P * 256-byte contiguous K / V slab read with 16-byte loads
// (16 lanes per token row), dot products use packed 16-bit dot instructions with fp32
// accumulation, and the softmax is kept online per wavefront.
//
// Work distribution: a launch is only a few thousand pages, far too few for the hardware scheduler
// to even out, so the page lists of all (sequence, KV head) pairs are laid end to end and cut into
// G equal ranges, G = resident workgroups of the whole chip.  A workgroup resolves the table entries
// of its pages in one go (one lane per page) and then streams its pages, the next page's slabs in
// flight while it works on the current one; its four wavefronts each take a quarter of a page's
// tokens.  A range may cross list boundaries; every (workgroup, list) piece yields either the final
// result (the list lies inside the range) or a partial (max, sum, unnormalised output) at slot
// workgroup + list index; the workgroup that delivers the last piece of a list folds them in slot order.
// Reduction orders are fixed, so results are deterministic.
//
// Pages may also hold quantised rows (Sec. 3.2: 8- or 4-bit codes with one fp16 scale and zero point per
// token, stored after the page's rows).  The kernel is the same with the slab loads and the per-page
// arithmetic swapped (template parameter BITS); see process_quantised_quarter_page.
#include <algorithm>

#include "kernels.h"

namespace lserve {

namespace {

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = kDecodeThreads / kWave;
constexpr int kMaxBlocksPerCU = 4;       // upper bound used to size the workspace
constexpr int kBlocksPerCU = 2;          // measured best on MI355X: more resident workgroups only queue up in the fabric
constexpr int kSlackFromEntries = 8;     // ranges at least this long model the cost of a list boundary (see make_plan)
constexpr float kLn2 = 0.6931471805599453f;

// ---- index tables --------------------------------------------------------------------------------

struct PageList {
    int len;          // number of pages attended
    int head;         // entries [0, head) come from `first`, the rest are consecutive from `tail_start`
    int tail_start;
    const int* first; // selected pages (NULL for streaming heads: entry i is page i)
};

// Index table of KV head hk (Sec. 3.6): streaming heads list sink and local pages, dense heads the
// selection followed by every page created after it.
__device__ __forceinline__ PageList make_page_list(const LayerParams& lp, int b, int hk, int L,
                                                   const int* sel_pages, const int* sel_count,
                                                   const int* sel_seq_len, int sel_stride) {
    PageList pl;
    const int P = ceil_div(L, lp.NP);
    if ((lp.streaming_mask >> hk) & 1ull) {
        pl.head = min(lp.sink_pages, P);
        pl.tail_start = max(pl.head, P - lp.local_pages);
        pl.first = nullptr;
    } else {
        pl.head = sel_count[b * lp.Hkv + hk];
        pl.tail_start = ceil_div(sel_seq_len[b], lp.NP);
        pl.first = sel_pages + ((size_t)b * lp.Hkv + hk) * sel_stride;
    }
    pl.len = pl.head + max(0, P - pl.tail_start);
    return pl;
}

__device__ __forceinline__ int page_of(const PageList& pl, int i) {
    if (i < pl.head) return pl.first ? pl.first[i] : i;
    return pl.tail_start + (i - pl.head);
}

// ---- per-wave online softmax over quarter pages --------------------------------------------------
//
// A wave owns NP / 4 consecutive tokens of every page.  Keys and values use different lane maps:
//   keys  : LPT lanes per token; lane l reads 16-byte chunks LPT * j + l % LPT of token l / LPT, so a
//           dot product over the 128 channels needs only log2(LPT) cross-lane steps (LPT = 4 for
//           N_P >= 64: every 4 lanes read 64 contiguous bytes);
//   values: 16 lanes per token row, lane (r, c) reads chunk c of tokens 4 it + r, so the output
//           accumulators stay at 8 channels per lane and head.
// The softmax weights cross from one map to the other through a few hundred bytes of LDS.

template <int NP> struct KeyMap {
    static constexpr int LPT = NP >= 64 ? 4 : (NP == 32 ? 8 : 16);  // lanes per token
    static constexpr int TPP = kWave / LPT;                          // tokens per pass of the wave
    static constexpr int PASSES = (NP / 4) / TPP;                    // 2 for N_P = 128, else 1
    static constexpr int KLOADS = 16 / LPT;                          // 16-byte chunks per lane and token
    static constexpr int ITS = NP / 16;                              // 16-byte loads per lane and slab
};

template <int NP, int BITS> struct Slabs;
template <int NP> struct Slabs<NP, 16> {
    uint4 k[KeyMap<NP>::ITS], v[KeyMap<NP>::ITS];
};
// Quantised pages (N_P = 64 only): a token row is 128 one-byte codes.  The key map keeps four lanes per token,
// each with two 16-byte chunks; the value map keeps 16 lanes per token row, each with eight codes.  The
// (scale, zero) pairs of both the K and the V row of a token travel with the key map's lane of that token.
template <> struct Slabs<64, 8> {
    uint4 k[2];
    uint2 v[4];
    uint32_t ksz, vsz;
};
// 4-bit codes: a token row is 64 bytes, byte j of every 4-byte word holding channel 8 g + j in its low and
// channel 8 g + 4 + j in its high half (g = index of the word).  One 16-byte chunk per key lane, one word per
// value lane.
template <> struct Slabs<64, 4> {
    uint4 k[1];
    uint32_t v[4];
    uint32_t ksz, vsz;
};

template <int NP>
__device__ __forceinline__ void load_k(Slabs<NP, 16>& s, const uint4* kslab, int tok0, int lane) {
    using M = KeyMap<NP>;
#pragma unroll
    for (int ps = 0; ps < M::PASSES; ++ps)
#pragma unroll
        for (int j = 0; j < M::KLOADS; ++j)
            s.k[ps * M::KLOADS + j] =
                kslab[(size_t)(tok0 + ps * M::TPP + lane / M::LPT) * (kHeadDim / 8) + M::LPT * j + lane % M::LPT];
}

template <int NP>
__device__ __forceinline__ void load_v(Slabs<NP, 16>& s, const uint4* vslab, int tok0, int r, int c, int) {
#pragma unroll
    for (int it = 0; it < KeyMap<NP>::ITS; ++it) s.v[it] = vslab[(size_t)(tok0 + 4 * it + r) * (kHeadDim / 8) + c];
}

__device__ __forceinline__ void load_k(Slabs<64, 4>& s, const uint4* kslab, int tok0, int lane) {
    const int tok = tok0 + lane / 4;
    s.k[0] = kslab[(size_t)tok * (kHeadDim / 32) + lane % 4];
    s.ksz = reinterpret_cast<const uint32_t*>(kslab + 64 * (kHeadDim / 32))[tok];
}
__device__ __forceinline__ void load_v(Slabs<64, 4>& s, const uint4* vslab, int tok0, int r, int c, int lane) {
    const uint32_t* rows = reinterpret_cast<const uint32_t*>(vslab);
#pragma unroll
    for (int it = 0; it < 4; ++it) s.v[it] = rows[(size_t)(tok0 + 4 * it + r) * (kHeadDim / 8) + c];
    s.vsz = reinterpret_cast<const uint32_t*>(vslab + 64 * (kHeadDim / 32))[tok0 + lane / 4];
}
__device__ __forceinline__ void load_k(Slabs<64, 8>& s, const uint4* kslab, int tok0, int lane) {
    const int tok = tok0 + lane / 4;
#pragma unroll
    for (int j = 0; j < 2; ++j) s.k[j] = kslab[(size_t)tok * (kHeadDim / 16) + 4 * j + lane % 4];
    s.ksz = reinterpret_cast<const uint32_t*>(kslab + 64 * (kHeadDim / 16))[tok];
}
__device__ __forceinline__ void load_v(Slabs<64, 8>& s, const uint4* vslab, int tok0, int r, int c, int lane) {
    const uint2* rows = reinterpret_cast<const uint2*>(vslab);
#pragma unroll
    for (int it = 0; it < 4; ++it) s.v[it] = rows[(size_t)(tok0 + 4 * it + r) * (kHeadDim / 8) + c];
    s.vsz = reinterpret_cast<const uint32_t*>(vslab + 64 * (kHeadDim / 16))[tok0 + lane / 4];
}

template <int N> struct WaveState {
    float m[N], l[N], o[N][8];
    float z[N];  // quantised values only: sum of weight * zero point, the same for every channel
    // Quantised pages keep the softmax of a token in the four lanes that read its key, one query head (two for
    // groups above four) per lane: lane l of a wave owns heads l % 4 and l % 4 + 4.  Running maximum, sum of weights
    // and zero-point sum of those heads; w_sum: per head, the sum of the 16-bit weights this lane fed to `o`.
    static constexpr int kHeadsPerLane = (N + 3) / 4;
    float lane_m[kHeadsPerLane], lane_l[kHeadsPerLane], lane_z[kHeadsPerLane], w_sum[N];
    __device__ __forceinline__ void reset() {
#pragma unroll
        for (int hh = 0; hh < N; ++hh) {
            m[hh] = -INFINITY;
            l[hh] = 0.f;
            z[hh] = 0.f;
            w_sum[hh] = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[hh][i] = 0.f;
        }
#pragma unroll
        for (int g = 0; g < kHeadsPerLane; ++g) {
            lane_m[g] = -INFINITY;
            lane_l[g] = 0.f;
            lane_z[g] = 0.f;
        }
    }
};

constexpr int p_row(int n) { return n <= 4 ? 4 : 8; }  // floats per token row of the weight buffer

// Sum over the LPT lanes that share a token; every one of them receives the total.
template <int LPT> __device__ __forceinline__ float token_sum(float x) {
    x += dpp_f<kDppXor1>(x);
    x += dpp_f<kDppXor2>(x);
    if (LPT >= 8) x += dpp_f<kDppHalfMirror>(x);
    if (LPT >= 16) x += dpp_f<kDppMirror>(x);
    return x;
}

// Maximum over the wave of a value that is already equal inside every group of four lanes.
__device__ __forceinline__ float wave_max_of_quads(float x) {
    x = fmaxf(x, dpp_f<kDppHalfMirror>(x));
    x = fmaxf(x, dpp_f<kDppMirror>(x));
    return rows4_max(x);
}

// One quarter page.  q_lds: [N][16] 16-byte chunks of the group's queries; p_lds: this wave's
// [NP / 4][p_row(N)] weight buffer.  `valid` = tokens of the page below the sequence length.
template <class T, int N, int NP>
__device__ __forceinline__ void process_quarter_page(WaveState<N>& st, const uint4* q_lds, const float*, float* p_lds,
                                                     Slabs<NP, 16>& cur, int valid, int tok0, int lane,
                                                     float scale_log2) {
    using M = KeyMap<NP>;
    constexpr int PR = p_row(N);
    const int r = lane / 16;
    float s[M::PASSES][N];
#pragma unroll
    for (int ps = 0; ps < M::PASSES; ++ps)
#pragma unroll
        for (int hh = 0; hh < N; ++hh) s[ps][hh] = 0.f;
#pragma unroll
    for (int j = 0; j < M::KLOADS; ++j) {
#pragma unroll
        for (int hh = 0; hh < N; ++hh) {
            const uint4 qv = q_lds[hh * 16 + M::LPT * j + lane % M::LPT];
            const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
            for (int ps = 0; ps < M::PASSES; ++ps) {
                const uint4 kv4 = cur.k[ps * M::KLOADS + j];
                const uint32_t kw[4] = {kv4.x, kv4.y, kv4.z, kv4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) s[ps][hh] = Elem<T>::dot2(qw[i], kw[i], s[ps][hh]);
            }
        }
    }
    const bool tail = valid < NP;
#pragma unroll
    for (int ps = 0; ps < M::PASSES; ++ps) {
        const bool dead = tail && tok0 + ps * M::TPP + lane / M::LPT >= valid;
#pragma unroll
        for (int hh = 0; hh < N; ++hh) {
            const float x = token_sum<M::LPT>(s[ps][hh]) * scale_log2;
            s[ps][hh] = dead ? -INFINITY : x;
        }
    }
#pragma unroll
    for (int hh = 0; hh < N; ++hh) {
        float pm = s[0][hh];
#pragma unroll
        for (int ps = 1; ps < M::PASSES; ++ps) pm = fmaxf(pm, s[ps][hh]);
        pm = wave_max_of_quads(pm);
        if (pm > st.m[hh]) {  // wave-uniform: rescale only when the running maximum moves
            const float alpha = __builtin_amdgcn_exp2f(st.m[hh] - pm);
            st.m[hh] = pm;
            st.l[hh] *= alpha;
            st.z[hh] *= alpha;
#pragma unroll
            for (int i = 0; i < 8; ++i) st.o[hh][i] *= alpha;
        }
        const float m_safe = st.m[hh] == -INFINITY ? 0.f : st.m[hh];
#pragma unroll
        for (int ps = 0; ps < M::PASSES; ++ps) {
            s[ps][hh] = __builtin_amdgcn_exp2f(s[ps][hh] - m_safe);
            st.l[hh] += s[ps][hh];  // counted once per lane of the token: divided by LPT at the end
        }
    }
    if (lane % M::LPT == 0) {
#pragma unroll
        for (int ps = 0; ps < M::PASSES; ++ps) {
            float* dst = p_lds + (ps * M::TPP + lane / M::LPT) * PR;
#pragma unroll
            for (int hh = 0; hh < N; ++hh) dst[hh] = s[ps][hh];
        }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < M::ITS; ++it) {
        uint4 vv = cur.v[it];
        if (tail && tok0 + 4 * it + r >= valid) vv = make_uint4(0, 0, 0, 0);  // slots past the end may hold anything
        const uint32_t vw[4] = {vv.x, vv.y, vv.z, vv.w};
        float pv[PR];
#pragma unroll
        for (int x4 = 0; x4 < PR / 4; ++x4) {
            const float4 t4 = *reinterpret_cast<const float4*>(p_lds + (4 * it + r) * PR + 4 * x4);
            pv[4 * x4] = t4.x;
            pv[4 * x4 + 1] = t4.y;
            pv[4 * x4 + 2] = t4.z;
            pv[4 * x4 + 3] = t4.w;
        }
#pragma unroll
        for (int hh = 0; hh < N; ++hh) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                st.o[hh][2 * i] = __builtin_fmaf(pv[hh], Elem<T>::lo(vw[i]), st.o[hh][2 * i]);
                st.o[hh][2 * i + 1] = __builtin_fmaf(pv[hh], Elem<T>::hi(vw[i]), st.o[hh][2 * i + 1]);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Value of lane k of the caller's group of four lanes.
__device__ __forceinline__ float quad_lane(float x, int k) {
    switch (k) {
        case 0: return dpp_f<0x00>(x);
        case 1: return dpp_f<0x55>(x);
        case 2: return dpp_f<0xAA>(x);
        default: return dpp_f<0xFF>(x);
    }
}

// Sums x0 .. x3 over the four lanes that share a token; lane k of the four receives the total of x_k.
__device__ __forceinline__ float quad_sum_scatter(float x0, float x1, float x2, float x3, int lane) {
    const bool odd = lane & 1, upper = lane & 2;
    float a0 = odd ? x1 : x0, a1 = odd ? x3 : x2;
    const float b0 = odd ? x0 : x1, b1 = odd ? x2 : x3;
    a0 += dpp_f<kDppXor1>(b0);
    a1 += dpp_f<kDppXor1>(b1);
    const float keep = upper ? a1 : a0, send = upper ? a0 : a1;
    return keep + dpp_f<kDppXor2>(send);
}

// Maximum over the sixteen lanes of a wave that have the caller's lane % 4; all of them receive it.
__device__ __forceinline__ float wave_max_same_quarter(float x) {
    x = fmaxf(x, dpp_f<0x124>(x));  // row_ror:4
    x = fmaxf(x, dpp_f<0x128>(x));  // row_ror:8
    return rows4_max(x);
}

constexpr float kWeightScale = 64.f;  // keeps weight * scale clear of the fp16 subnormals, and below 65504 for any fp16 row

// The same over a quantised quarter page.  q_lds holds the queries as fp16 whatever the storage type and
// q_sum[h] the sum of query h's channels.  With k = code * scale + zero the logit of a token is
//   q . k = scale * (q . code) + zero * sum(q).
// Codes become fp16 without a conversion: byte c under the exponent byte 0x64 is the fp16 number 1024 + c,
// so one byte permute yields two operands of the packed dot instruction, and the 1024 * sum(q) this adds
// to every dot product is taken off again.  For values the weight is folded into the scale,
//   sum_t p_t v_t = sum_t (p_t scale_t) code_t + sum_t p_t zero_t,
// and the second sum, which no channel distinguishes, is kept as one number per query head.
//
// The instruction count, not the memory system, bounds this path (a page is half or a quarter of the bytes for the
// same number of tokens), so it is arranged to issue as little as possible per token:
//   - after the dot products the four lanes of a token hold four partial sums for each of N heads; a reduce-scatter
//     leaves lane k with the total of head k, and maximum, exponential, sums and scales are then computed once
//     per (token, head) instead of four times;
//   - the weights go to LDS as fp16 (times kWeightScale), two tokens of a value row side by side, so that the
//     value side reads ready-made pairs and takes two tokens per packed dot instruction, with the codes of the
//     two tokens interleaved by byte permutes and lifted to 1024 + code like the keys; the 1024 * (sum of the
//     rounded weights) this adds to every channel is subtracted, and the scale undone, once per piece of a list
//     (lane_state_to_wave_state).  A weight is rounded to fp16 (2^-11 relative) before it meets the codes; the
//     denominator keeps the unrounded weights.
// p_lds is read as 16-bit [token pair][value row r][p_row(N) heads][2 tokens].
template <class T, int N, int BITS>
__device__ __forceinline__ void process_quantised_quarter_page(WaveState<N>& st, const uint4* q_lds, const float* q_sum,
                                                     float* p_lds, Slabs<64, BITS>& cur, int valid, int tok0, int lane,
                                                     float scale_log2) {
    static_assert(BITS == 8 || BITS == 4, "quantised pages");
    constexpr int PR = p_row(N), HPL = WaveState<N>::kHeadsPerLane;
    const int r = lane / 16, qd = lane % 4;
    float s[4 * HPL];
#pragma unroll
    for (int hh = 0; hh < 4 * HPL; ++hh) s[hh] = 0.f;
    // 16 channels at a time: four bytes-per-code words (two of the 8-bit chunk's words, or the low and the high
    // halves of two of the 4-bit chunk's words) become eight fp16 pairs and meet two 8-channel query chunks
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        uint32_t kw[4];
        int qc;  // first of the two query chunks
        if constexpr (BITS == 8) {
            kw[0] = cur.k[j].x, kw[1] = cur.k[j].y, kw[2] = cur.k[j].z, kw[3] = cur.k[j].w;
            qc = 2 * (4 * j + lane % 4);  // 16-byte chunk 4 j + lane % 4 of the row = channels 16 cb .. 16 cb + 15
        } else {
            const uint32_t w0 = j == 0 ? cur.k[0].x : cur.k[0].z, w1 = j == 0 ? cur.k[0].y : cur.k[0].w;
            kw[0] = w0 & 0x0f0f0f0fu, kw[1] = (w0 >> 4) & 0x0f0f0f0fu;  // channels 8 g .. 8 g + 3, 8 g + 4 .. 8 g + 7
            kw[2] = w1 & 0x0f0f0f0fu, kw[3] = (w1 >> 4) & 0x0f0f0f0fu;
            qc = 4 * (lane % 4) + 2 * j;  // word g = 4 (lane % 4) + 2 j + {0, 1} of the row = channels 8 g .. 8 g + 7
        }
        uint32_t kh[8];  // 16 codes as eight fp16 pairs (1024 + code)
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            kh[2 * d] = __builtin_amdgcn_perm(0x64646464u, kw[d], 0x04010400u);
            kh[2 * d + 1] = __builtin_amdgcn_perm(0x64646464u, kw[d], 0x04030402u);
        }
#pragma unroll
        for (int hh = 0; hh < N; ++hh) {
            const uint4 qa = q_lds[hh * 16 + qc], qb = q_lds[hh * 16 + qc + 1];
            const uint32_t qw[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
#pragma unroll
            for (int u = 0; u < 8; ++u) s[hh] = Elem<F16>::dot2(qw[u], kh[u], s[hh]);
        }
    }
    const bool dead = valid < 64 && tok0 + lane / 4 >= valid;
    const half2_t ksz = __builtin_bit_cast(half2_t, cur.ksz), vsz = __builtin_bit_cast(half2_t, cur.vsz);
    const float k_scale = (float)ksz[0] * scale_log2, k_zero = (float)ksz[1] * scale_log2;
    // slots past the end may hold anything
    const float v_scale = dead ? 0.f : (float)vsz[0] * kWeightScale, v_zero = dead ? 0.f : (float)vsz[1];
    // this lane's place in the weight buffer: token lane / 4 of the quarter page is member (t / 4) % 2 of pair t / 8 of
    // value row t % 4
    const int t = lane / 4;
    _Float16* w_lds = reinterpret_cast<_Float16*>(p_lds) + (((t / 8) * 4 + t % 4) * PR + qd) * 2 + (t / 4) % 2;
#pragma unroll
    for (int g = 0; g < HPL; ++g) {
        const bool mine = 4 * g + qd < N;  // lanes without a head of their own carry zeros along
        const float qs = mine ? q_sum[4 * g + qd] : 0.f;
        const float dot = quad_sum_scatter(s[4 * g], s[4 * g + 1], s[4 * g + 2], s[4 * g + 3], lane) - 1024.f * qs;
        const float x = dead ? -INFINITY : __builtin_fmaf(k_scale, dot, k_zero * qs);
        const float pm = wave_max_same_quarter(x);
        const bool moved = pm > st.lane_m[g];
        if (__any(moved)) {  // rare after the first pages: some head's running maximum moves
            const float alpha = moved ? __builtin_amdgcn_exp2f(st.lane_m[g] - pm) : 1.f;
            st.lane_m[g] = moved ? pm : st.lane_m[g];
            st.lane_l[g] *= alpha;
            st.lane_z[g] *= alpha;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (4 * g + k >= N) continue;
                const float a = quad_lane(alpha, k);
                st.w_sum[4 * g + k] *= a;
#pragma unroll
                for (int i = 0; i < 8; ++i) st.o[4 * g + k][i] *= a;
            }
        }
        const float m_safe = st.lane_m[g] == -INFINITY ? 0.f : st.lane_m[g];
        const float p = dead ? 0.f : __builtin_amdgcn_exp2f(x - m_safe);
        st.lane_l[g] += p;
        st.lane_z[g] = __builtin_fmaf(p, v_zero, st.lane_z[g]);
        w_lds[8 * g] = (_Float16)(p * v_scale);  // head 4 g + qd: four heads = four token pairs = eight halves on
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
        uint32_t ta[2], tb[2];  // one byte per code, channels 0 .. 3 and 4 .. 7 of the pair's two tokens
        if constexpr (BITS == 8) {
            ta[0] = cur.v[2 * pr].x, ta[1] = cur.v[2 * pr].y;
            tb[0] = cur.v[2 * pr + 1].x, tb[1] = cur.v[2 * pr + 1].y;
        } else {
            ta[0] = cur.v[2 * pr] & 0x0f0f0f0fu, ta[1] = (cur.v[2 * pr] >> 4) & 0x0f0f0f0fu;
            tb[0] = cur.v[2 * pr + 1] & 0x0f0f0f0fu, tb[1] = (cur.v[2 * pr + 1] >> 4) & 0x0f0f0f0fu;
        }
        uint32_t wp[PR];  // (weight of the first token, weight of the second) per head, fp16
#pragma unroll
        for (int x4 = 0; x4 < PR / 4; ++x4) {
            const uint4 w4 = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint32_t*>(p_lds) + (pr * 4 + r) * PR + 4 * x4);
            wp[4 * x4] = w4.x, wp[4 * x4 + 1] = w4.y, wp[4 * x4 + 2] = w4.z, wp[4 * x4 + 3] = w4.w;
        }
        uint32_t ch[8];  // channel i of both tokens as an fp16 pair (1024 + code)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t lo = __builtin_amdgcn_perm(tb[u], ta[u], 0x05010400u);  // a0 b0 a1 b1
            const uint32_t hi = __builtin_amdgcn_perm(tb[u], ta[u], 0x07030602u);  // a2 b2 a3 b3
            ch[4 * u] = __builtin_amdgcn_perm(0x64646464u, lo, 0x04010400u);
            ch[4 * u + 1] = __builtin_amdgcn_perm(0x64646464u, lo, 0x04030402u);
            ch[4 * u + 2] = __builtin_amdgcn_perm(0x64646464u, hi, 0x04010400u);
            ch[4 * u + 3] = __builtin_amdgcn_perm(0x64646464u, hi, 0x04030402u);
        }
#pragma unroll
        for (int hh = 0; hh < N; ++hh) {
            st.w_sum[hh] = Elem<F16>::dot2(wp[hh], 0x3c003c00u, st.w_sum[hh]);
#pragma unroll
            for (int i = 0; i < 8; ++i) st.o[hh][i] = Elem<F16>::dot2(wp[hh], ch[i], st.o[hh][i]);
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Turns the per-lane softmax state of the quantised path into the form flush_block() folds: per head a wave-uniform
// maximum, per-lane sums that add up (over the wave) to four times the head's total, and outputs with the code
// offset and the weight scale taken off.
template <int N>
__device__ __forceinline__ void lane_state_to_wave_state(WaveState<N>& st, int lane) {
    const int qd = lane % 4;
#pragma unroll
    for (int hh = 0; hh < N; ++hh) {
        const int g = hh / 4, k = hh % 4;
        st.m[hh] = quad_lane(st.lane_m[g], k);
        st.l[hh] = qd == k ? 4.f * st.lane_l[g] : 0.f;
        st.z[hh] = qd == k ? 4.f * st.lane_z[g] : 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            st.o[hh][i] = __builtin_fmaf(-1024.f, st.w_sum[hh], st.o[hh][i]) * (1.f / kWeightScale);
    }
}

template <class T, int N, int NP, int BITS>
__device__ __forceinline__ void process_quarter(WaveState<N>& st, const uint4* q_lds, const float* q_sum, float* p_lds,
                                                Slabs<NP, BITS>& cur, int valid, int tok0, int lane, float scale_log2) {
    if constexpr (BITS == 16)
        process_quarter_page<T, N, NP>(st, q_lds, q_sum, p_lds, cur, valid, tok0, lane, scale_log2);
    else
        process_quantised_quarter_page<T, N, BITS>(st, q_lds, q_sum, p_lds, cur, valid, tok0, lane, scale_log2);
}

// Shared memory of a decode workgroup.
template <int N, int NP> struct DecodeShared {
    float o[kDecodeWaves][N][kHeadDim];   // cross-wave merge
    float m[kDecodeWaves][N], l[kDecodeWaves][N], z[kDecodeWaves][N];
    uint4 q[N * 16];                      // queries of the current group
    float q_sum[kMaxGroup];               // quantised pages only: sum over the channels of each query
    float p[kDecodeWaves][(NP / 4) * p_row(N)];
    unsigned arrived;                     // pieces of a cut list that were in before this workgroup's
};

// Loads the n queries of KV head hk into shared memory.  Called by the whole workgroup.
// For quantised pages the queries are converted to fp16 (exact for every bf16 value of magnitude between
// 2^-14 and 65504; larger ones saturate) and their channel sums are taken, from the converted values.
// A workgroup's range starts inside a list that is known from the launch plan alone, so the queries of that
// list and of the one after it are requested at the very start of the kernel, in parallel with the table
// look-ups, and are at hand when the first page (or the first page after a list boundary) arrives: the load
// would otherwise sit exposed between two workgroup barriers.
struct QueryAhead {
    int list;      // first list of the range; list + 1 is held too
    uint4 x[2];    // this thread's 16-byte chunk of the group's queries (threads below N * 16)
};

template <class T, int N, int NP, int BITS>
__device__ __forceinline__ void stage_query(DecodeShared<N, NP>& sm, const uint4* q, int b, int H, int hk, int list,
                                            const QueryAhead& ahead) {
    static_assert(N * 16 <= kDecodeThreads, "one pass");
    const int i = threadIdx.x;  // chunk i of the group: the 16 chunks of a query are the 16 lanes of a DPP row
    uint4 x = ahead.x[0];
    if (list == ahead.list + 1) x = ahead.x[1];
    if ((list < ahead.list || list > ahead.list + 1) && i < N * 16) x = q[((size_t)b * H + hk * N) * (kHeadDim / 8) + i];
    __syncthreads();  // earlier readers of sm.q are done
    if (BITS == 16) {
        if (i < N * 16) sm.q[i] = x;
    } else {
        float part = 0.f;
        if (i < N * 16) {
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
            uint32_t o[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float a = fminf(fmaxf(Elem<T>::lo(w[u]), -65504.f), 65504.f);
                const float c = fminf(fmaxf(Elem<T>::hi(w[u]), -65504.f), 65504.f);
                o[u] = Elem<F16>::pack(a, c);
                part += Elem<F16>::lo(o[u]) + Elem<F16>::hi(o[u]);
            }
            sm.q[i] = make_uint4(o[0], o[1], o[2], o[3]);
        }
        part = row16_sum(part);
        if (i < N * 16 && i % 16 == 0) sm.q_sum[i / 16] = part;
    }
    __syncthreads();
}

// Partial results travel between workgroups that may sit on different XCDs, each with an L2 of its own.  They are
// written and read with agent-scope accesses (write-through stores, loads that are not served from a stale line),
// which costs those few hundred kilobytes nothing, instead of fences that write back and invalidate whole caches.
// Two floats per access (8-byte aligned).
__device__ __forceinline__ void store_shared_across_chip(float* p, float a, float b) {
    const float2 v = make_float2(a, b);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_shared_across_chip(const float* p) {
    return __builtin_bit_cast(float2, __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT));
}

// Folds the four token rows of every wave, then the four waves of the workgroup, and writes either
// the final rows (out / lse) or a partial (part_o / part_ml).  Must be called by all 256 threads.
template <class T, int N, int NP, int BITS>
__device__ __forceinline__ void flush_block(WaveState<N>& st, DecodeShared<N, NP>& sm, bool final_result, int H,
                                            int b, int hk, uint16_t* out, float* lse_out, float* part_o,
                                            float* part_ml, size_t part_slot) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int r = lane / 16, c = lane % 16;
    // Sums over the four token rows of the wave, four values at a time: row r ends up with the total of the r-th.
    constexpr int kQuads = (N + 3) / 4;
    float lrow[4 * kQuads], zrow[4 * kQuads];
#pragma unroll
    for (int hh = 0; hh < 4 * kQuads; ++hh) {
        // every lane of a token added the token's weight (and, for quantised values, its share of the zero-point
        // term, which belongs to every channel): the 64 lanes hold LPT copies of each sum
        lrow[hh] = hh < N ? row16_sum(st.l[hh]) : 0.f;
        zrow[hh] = hh < N && BITS != 16 ? row16_sum(st.z[hh]) : 0.f;
    }
#pragma unroll
    for (int g = 0; g < kQuads; ++g) {
        const float lsum = rows4_sum_scatter(lrow[4 * g], lrow[4 * g + 1], lrow[4 * g + 2], lrow[4 * g + 3]);
        float zsum = 0.f;
        if (BITS != 16) zsum = rows4_sum_scatter(zrow[4 * g], zrow[4 * g + 1], zrow[4 * g + 2], zrow[4 * g + 3]);
        if (c == 0 && 4 * g + r < N) {
            sm.l[wave][4 * g + r] = lsum * (1.0f / KeyMap<NP>::LPT);
            sm.z[wave][4 * g + r] = zsum * (1.0f / KeyMap<NP>::LPT);
        }
    }
#pragma unroll
    for (int hh = 0; hh < N; ++hh) {
#pragma unroll
        for (int g = 0; g < 2; ++g)  // lane (r, c) receives channel 8 c + 4 g + r
            sm.o[wave][hh][8 * c + 4 * g + r] =
                rows4_sum_scatter(st.o[hh][4 * g], st.o[hh][4 * g + 1], st.o[hh][4 * g + 2], st.o[hh][4 * g + 3]);
        if (lane == 0) sm.m[wave][hh] = st.m[hh];
    }
    __syncthreads();
    // one thread per (query head, four channels): N * 32 <= 256 work items
    if (threadIdx.x < N * (kHeadDim / 4)) {
        const int hh = threadIdx.x / (kHeadDim / 4), ch = threadIdx.x % (kHeadDim / 4) * 4;
        float M = sm.m[0][hh];
#pragma unroll
        for (int w = 1; w < kDecodeWaves; ++w) M = fmaxf(M, sm.m[w][hh]);
        float lt = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            const float f = sm.m[w][hh] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sm.m[w][hh] - M);
            lt += sm.l[w][hh] * f;
            const float4 o4 = *reinterpret_cast<const float4*>(&sm.o[w][hh][ch]);
            const float z = BITS != 16 ? sm.z[w][hh] : 0.f;
            acc[0] += (o4.x + z) * f;
            acc[1] += (o4.y + z) * f;
            acc[2] += (o4.z + z) * f;
            acc[3] += (o4.w + z) * f;
        }
        const int h = hk * N + hh;
        if (final_result) {
            const uint2 packed = make_uint2(Elem<T>::pack(acc[0] / lt, acc[1] / lt), Elem<T>::pack(acc[2] / lt, acc[3] / lt));
            *reinterpret_cast<uint2*>(out + ((size_t)b * H + h) * kHeadDim + ch) = packed;
            if (lse_out && ch == 0) lse_out[b * H + h] = (M + __builtin_amdgcn_logf(lt)) * kLn2;
        } else {
            const size_t pi = part_slot * N + hh;
            store_shared_across_chip(part_o + pi * kHeadDim + ch, acc[0], acc[1]);
            store_shared_across_chip(part_o + pi * kHeadDim + ch + 2, acc[2], acc[3]);
            if (ch == 0) store_shared_across_chip(part_ml + pi * 2, M, lt);
        }
    }
    __syncthreads();
}

// ---- balanced kernel over the nominal page space -------------------------------------------------
//
// Launch shape and work split must not depend on device data, and a prefix sum over the real list
// lengths would put two more dependent memory round trips in front of the first K/V load of every
// workgroup.  The split is therefore done over *nominal* list lengths the host knows: s + w pages
// for a streaming head, sel_stride + 1 for a dense head (the selection plus one page created since).
// Nominal entry x of the launch maps to (sequence, KV head, entry) by arithmetic alone.  Entries
// past a list's real length are skipped; real entries past the nominal length (a selection reused
// for more than one new page) are handled by the workgroup that owns the list's last nominal entry.

struct DecodePlan {
    int per_seq;                 // nominal entries per sequence
    int total;                   // batch * per_seq
    int quot, rem;               // total = G * quot + rem: the first `rem` ranges hold quot + 1 entries
    int stream_len, select_len;  // nominal entries of a streaming head's list and of a selecting head's
};

// First nominal entry of KV head hk inside a sequence (hk = Hkv gives per_seq).  The lists of a sequence follow
// each other in head order, so the start is a count of the streaming heads below hk: plain arithmetic on two
// launch constants, with nothing to fetch before the first table look-up can be issued.
__device__ __forceinline__ int first_entry(const DecodePlan& plan, unsigned long long streaming_mask, int hk) {
    const unsigned long long below = hk >= 64 ? ~0ull : (1ull << hk) - 1ull;
    const int ns = __popcll(streaming_mask & below);
    return ns * plan.stream_len + (hk - ns) * plan.select_len;
}
__device__ __forceinline__ int nominal_len(const DecodePlan& plan, unsigned long long streaming_mask, int hk) {
    return ((streaming_mask >> hk) & 1ull) ? plan.stream_len : plan.select_len;
}

// Range of workgroup j is [range_begin(j), range_begin(j + 1)); no division on the device.
__device__ __forceinline__ int range_begin(const DecodePlan& plan, int j) { return j * plan.quot + min(j, plan.rem); }

// Workgroup whose range holds nominal entry x.
__device__ __forceinline__ int range_of(const DecodePlan& plan, int x) {
    const int big = plan.rem * (plan.quot + 1);
    return x < big ? x / (plan.quot + 1) : plan.rem + (x - big) / plan.quot;
}

// KV head of nominal entry y of a sequence: the number of heads whose list starts at or before y, less one.
__device__ __forceinline__ int head_of_entry(const DecodePlan& plan, unsigned long long streaming_mask, int Hkv, int y) {
    int hk = 0;
    for (int h = 1; h < Hkv; ++h) hk += y >= first_entry(plan, streaming_mask, h);
    return hk;
}

// Folds the pieces of one list, in slot order, kBatch at a time so that their loads are in flight together, for
// four channels `ch .. ch + 3` of query head `hh` of the group.  Every range between j0 and j1 holds a real entry
// of the list and wrote a piece (ranges there are never empty: an empty range implies quot = 0, and then no list
// spans two ranges).
template <class T, int N, int kBatch>
__device__ __forceinline__ void fold_pieces(int list, int j0, int j1, int hh, int ch, int H, int b, int hk,
                                            uint16_t* out, float* lse_out, const float* part_o,
                                            const float* part_ml) {
    float M = -INFINITY, lt = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int jb = j0; jb <= j1; jb += kBatch) {
        float2 ml[kBatch], lo[kBatch], hi[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const size_t pi = ((size_t)min(jb + u, j1) + list) * N + hh;  // past the end: the last piece again, unused
            ml[u] = load_shared_across_chip(part_ml + pi * 2);
            lo[u] = load_shared_across_chip(part_o + pi * kHeadDim + ch);
            hi[u] = load_shared_across_chip(part_o + pi * kHeadDim + ch + 2);
        }
        float bm = -INFINITY;
#pragma unroll
        for (int u = 0; u < kBatch; ++u) bm = fmaxf(bm, jb + u <= j1 ? ml[u].x : -INFINITY);
        if (bm == -INFINITY) continue;  // only if every logit of these pieces was -inf
        const float m_new = fmaxf(M, bm);
        const float keep = __builtin_amdgcn_exp2f(M - m_new);  // 0 for the first batch (M = -inf)
        lt *= keep;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] *= keep;
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const float f = jb + u <= j1 ? __builtin_amdgcn_exp2f(ml[u].x - m_new) : 0.f;
            lt += ml[u].y * f;
            acc[0] += lo[u].x * f;
            acc[1] += lo[u].y * f;
            acc[2] += hi[u].x * f;
            acc[3] += hi[u].y * f;
        }
        M = m_new;
    }
    const int h = hk * N + hh;
    const uint2 packed = make_uint2(Elem<T>::pack(acc[0] / lt, acc[1] / lt), Elem<T>::pack(acc[2] / lt, acc[3] / lt));
    *reinterpret_cast<uint2*>(out + ((size_t)b * H + h) * kHeadDim + ch) = packed;
    if (lse_out && ch == 0) lse_out[b * H + h] = (M + __builtin_amdgcn_logf(lt)) * kLn2;
}

// Ends a (workgroup, list) piece.  `len` is the real length of the list, so its real entries occupy the nominal
// entries [n0, n_end) and exactly the workgroups whose ranges meet that stretch hold a piece of it.  A list that
// lies inside this workgroup's range is written out directly.  Otherwise the piece goes to the workspace, the
// workgroup counts itself in on the list's arrival counter, and the one that finds every other piece already in
// folds them all, in slot order (so the result does not depend on which workgroup folds), writes the rows and
// puts the counter back to zero for the next launch.  Nobody waits for anybody.  Stores, counter and loads are
// agent-scope accesses with a wait for the stores in between; no cache-wide fence (a device-scope fence here was
// measured at three times the whole kernel: it writes back and invalidates the L2).  Called by all threads.
template <class T, int N, int NP, int BITS>
__device__ __forceinline__ void end_piece(WaveState<N>& st, DecodeShared<N, NP>& sm, const DecodePlan& plan, int blk,
                                          int lo, int hi, int list, int len, int H, int Hkv,
                                          unsigned long long streaming_mask, uint16_t* out,
                                          float* lse_out, float* part_o, float* part_ml, unsigned* arrivals) {
    const int b = list / Hkv, hk = list % Hkv;
    const int n0 = b * plan.per_seq + first_entry(plan, streaming_mask, hk);
    const int n_end = n0 + min(len, nominal_len(plan, streaming_mask, hk));
    const bool whole = n0 >= lo && n_end <= hi;
    if constexpr (BITS != 16) lane_state_to_wave_state<N>(st, threadIdx.x % kWave);
    flush_block<T, N, NP, BITS>(st, sm, whole, H, b, hk, out, lse_out, part_o, part_ml, (size_t)blk + list);
    if (whole) return;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's part of the piece has reached memory
    __syncthreads();
    if (threadIdx.x == 0)
        sm.arrived = __hip_atomic_fetch_add(arrivals + list, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int j0 = range_of(plan, n0), j1 = range_of(plan, n_end - 1);
    if ((int)sm.arrived != j1 - j0) return;  // somebody else will fold
    if (threadIdx.x < N * (kHeadDim / 4))
        fold_pieces<T, N, 8>(list, j0, j1, threadIdx.x / (kHeadDim / 4), threadIdx.x % (kHeadDim / 4) * 4, H, b, hk, out,
                             lse_out, part_o, part_ml);
    if (threadIdx.x == 0) __hip_atomic_store(arrivals + list, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Visits entry IDX of the current batch, whose slabs are in CUR: when the (wave-uniform) list changes the
// piece of the previous list is ended and the new list's queries are staged; then the quarter page is
// folded in; real entries beyond the nominal length of a list (rare) are fetched and folded in on the spot,
// without prefetch (only dense heads outgrow their nominal list, so they are always in the main pool).
// A macro, not a lambda: with the state captured by reference the compiler keeps 70 more registers live in
// the 16-bit kernel.
#define LSERVE_DECODE_VISIT(IDX, CUR)                                                                                \
    {                                                                                                                \
        const int list = __builtin_amdgcn_readlane(my_list, (IDX));                                                  \
        if (list != cur_list) {                                                                                      \
            if (cur_list >= 0)                                                                                       \
                end_piece<T, N, NP, BITS>(st, sm, plan, blk, lo, hi, cur_list, cur_len, lp.H, lp.Hkv,                \
                                          lp.streaming_mask, out, lse_out, part_o, part_ml, arrivals);               \
            cur_list = list;                                                                                         \
            cur_len = __builtin_amdgcn_readlane(my_len, (IDX));                                                      \
            cur_b = list / lp.Hkv;                                                                                   \
            cur_hk = list % lp.Hkv;                                                                                  \
            stage_query<T, N, NP, BITS>(sm, q, cur_b, lp.H, cur_hk, list, q_ahead);                                  \
            st.reset();                                                                                              \
        }                                                                                                            \
        const int L = __builtin_amdgcn_readlane(my_L, (IDX));                                                        \
        const int pos = __builtin_amdgcn_readlane(my_pos, (IDX));                                                    \
        process_quarter<T, N, NP, BITS>(st, sm.q, sm.q_sum, sm.p[wave], CUR, L - pos * NP, tok0, lane, lp.sm_scale_log2); \
        const int extra = __builtin_amdgcn_readlane(my_extra, (IDX));                                                \
        if (extra > 0) {                                                                                             \
            const int nominal = nominal_len(plan, lp.streaming_mask, cur_hk);                                        \
            const int tail = __builtin_amdgcn_readlane(my_tail, (IDX));                                              \
            for (int e = 0; e < extra; ++e) {                                                                        \
                const int epos = tail + nominal + e;                                                                 \
                const int ephys = kv.page_table[(size_t)cur_b * kv.max_pages + epos];                                \
                const uint4 *ke, *ve;                                                                                \
                slab_of(ephys, cur_hk, ke, ve);                                                                      \
                load_k(CUR, ke, tok0, lane);                                                                         \
                load_v(CUR, ve, tok0, r, c, lane);                                                                   \
                process_quarter<T, N, NP, BITS>(st, sm.q, sm.q_sum, sm.p[wave], CUR, L - epos * NP, tok0, lane, lp.sm_scale_log2);\
            }                                                                                                        \
        }                                                                                                            \
    }

template <class T, int N, int NP, int BITS>
__global__ __launch_bounds__(kDecodeThreads) void sparse_decode_kernel(
    LayerParams lp, PagedParams kv, DecodePlan plan, const uint4* __restrict__ q, const int* __restrict__ sel_pages,
    const int* __restrict__ sel_count, const int* __restrict__ sel_seq_len, int sel_stride,
    uint16_t* __restrict__ out, float* __restrict__ lse_out, float* __restrict__ part_o, float* __restrict__ part_ml,
    unsigned* __restrict__ arrivals) {
    __shared__ DecodeShared<N, NP> sm;

    // The launch constants fill four 64-byte lines of the kernel argument block, and the code below wants them in
    // half a dozen dependent rounds; fetched as needed, each round missed the scalar cache and the first table
    // look-up left 2.2 us after the start of the kernel.  One word of every line is requested here, together.
#if defined(__HIP_DEVICE_COMPILE__)
    {
        typedef const int __attribute__((address_space(4))) * kernarg_words;
        const kernarg_words args = (kernarg_words)__builtin_amdgcn_kernarg_segment_ptr();
        static_assert(sizeof(LayerParams) + sizeof(PagedParams) + sizeof(DecodePlan) + 9 * sizeof(void*) > 48 * sizeof(int),
                      "the argument block must reach the last line touched");
        const int a0 = args[0], a1 = args[16], a2 = args[32], a3 = args[48];
        asm volatile("" ::"s"(a0), "s"(a1), "s"(a2), "s"(a3));
    }
#endif

    const int blk = blockIdx.x;
    const int lo = range_begin(plan, blk), hi = range_begin(plan, blk + 1);
    if (lo >= hi) return;

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int r = lane / 16, c = lane % 16;
    const int tok0 = wave * (NP / 4);
    const size_t slab = slab_chunks(NP, BITS);  // uint4 per (page, head)
    const uint4* kpool = reinterpret_cast<const uint4*>(kv.k_pool);
    const uint4* vpool = reinterpret_cast<const uint4*>(kv.v_pool);
    const uint4* kstream = reinterpret_cast<const uint4*>(kv.k_stream);
    const uint4* vstream = reinterpret_cast<const uint4*>(kv.v_stream);
    // slab of (physical page, KV head): streaming heads may live in their own bounded pool (Sec. 3.2)
    auto slab_of = [&](int phys, int hk, const uint4*& kslab, const uint4*& vslab) {
        const bool ring = in_stream_pool(lp, kv, hk);
        const size_t o = ((size_t)phys * (ring ? kv.stream_heads : kv.pool_heads) + pool_rank(lp, kv, hk, ring)) * slab;
        kslab = (ring ? kstream : kpool) + o;
        vslab = (ring ? vstream : vpool) + o;
    };

    // Only where the eight registers do not cost a resident workgroup (measured: 128-token pages and the
    // quantised kernels lose more than the early queries gain).
    constexpr bool kQueriesAhead = BITS == 16 && NP <= 64;
    QueryAhead q_ahead;
    q_ahead.list = -4;  // matches no list
    q_ahead.x[0] = q_ahead.x[1] = make_uint4(0, 0, 0, 0);

    WaveState<N> st;
    int cur_list = -1, cur_b = 0, cur_hk = 0, cur_len = 0;
    // with every head streaming there is no selection: the loads below then read a valid word of the lengths
    const int* sel_table = sel_pages ? sel_pages : kv.seq_lens;
    const int* sel_counts = sel_pages ? sel_count : kv.seq_lens;
    const int* sel_lens = sel_pages ? sel_seq_len : kv.seq_lens;
    const int has_sel = sel_pages != nullptr;  // a factor, not a condition: the loads must not sit behind a branch

    for (int base = lo; base < hi; base += kWave) {
        // One lane per nominal entry.  Every load that depends on nothing loaded goes out first and together (the
        // length; for a selecting head its selection entry, count and selection-time length), then the page
        // table, then the slabs: three round trips before the first byte of K / V, and no more.  Lanes past the
        // end of the range repeat its last entry, so that every lane forms valid addresses without a branch.
        const int cnt = min(kWave, hi - base);
        const int x = base + min(lane, cnt - 1);
        const int b = x / plan.per_seq, y = x - b * plan.per_seq;
        const int hk = head_of_entry(plan, lp.streaming_mask, lp.Hkv, y);
        const int i = y - first_entry(plan, lp.streaming_mask, hk), nominal = nominal_len(plan, lp.streaming_mask, hk);
        const bool streaming = (lp.streaming_mask >> hk) & 1ull;
        const int my_list = b * lp.Hkv + hk;
        // no branch between these loads and their first use, or the wait for them could not be counted exactly
        // and would take in the query loads as well; lanes of streaming heads read valid words they ignore
        const int my_L = kv.seq_lens[b];
        const int sel_word = sel_table[has_sel * ((size_t)my_list * sel_stride + min(i, sel_stride - 1))];
        const int sel_head = sel_counts[has_sel * my_list];
        const int sel_len = sel_lens[has_sel * b];
        // The queries of the first two lists of these entries go out behind the table loads (in front of them they
        // would be waited for first: loads complete in order).  Thread t holds chunk t % (N * 16) of the group.
        if constexpr (kQueriesAhead) {
            q_ahead.list = __builtin_amdgcn_readfirstlane(my_list);
            const int last = kv.batch * lp.Hkv - 1;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int list = min(q_ahead.list + u, last);
                q_ahead.x[u] = q[((size_t)(list / lp.Hkv) * lp.H + (list % lp.Hkv) * N) * (kHeadDim / 8) +
                                 threadIdx.x % (N * 16)];
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // all of the above is requested before any of it is used
        const int P = ceil_div(my_L, NP);
        const int stream_head = min(lp.sink_pages, P);
        const int head = streaming ? stream_head : sel_head;
        const int tail_start = streaming ? max(stream_head, P - lp.local_pages) : ceil_div(sel_len, NP);
        const int sel_entry = streaming ? i : sel_word;
        const int my_len = head + max(0, P - tail_start);
        const bool my_valid = lane < cnt && i < my_len;
        const int my_pos = i < head ? sel_entry : tail_start + (i - head);
        const int my_tail = tail_start - head;  // position of entry i >= head is my_tail + i
        const int my_extra = (i == nominal - 1 && my_len > nominal) ? my_len - nominal : 0;
        int my_phys = 0;
        if (my_valid)
            my_phys = in_stream_pool(lp, kv, hk) ? kv.ring_table[(size_t)b * kv.ring + ring_slot(lp, my_pos)]
                                                 : kv.page_table[(size_t)b * kv.max_pages + my_pos];
        unsigned long long todo = __ballot(my_valid);
        if (todo == 0) continue;
        if constexpr (BITS == 16) {
            // one page in flight behind the one being worked on
            Slabs<NP, BITS> cur, nxt;
            {
                const int idx0 = __builtin_ctzll(todo);
                const uint4 *k0, *v0;
                slab_of(__builtin_amdgcn_readlane(my_phys, idx0), __builtin_amdgcn_readlane(my_list, idx0) % lp.Hkv, k0, v0);
                load_k(cur, k0, tok0, lane);
                load_v(cur, v0, tok0, r, c, lane);
            }
            while (todo) {
                const int idx = __builtin_ctzll(todo);
                todo &= todo - 1;
                if (todo) {
                    const int idx1 = __builtin_ctzll(todo);
                    const uint4 *k1, *v1;
                    slab_of(__builtin_amdgcn_readlane(my_phys, idx1), __builtin_amdgcn_readlane(my_list, idx1) % lp.Hkv, k1, v1);
                    load_k(nxt, k1, tok0, lane);
                    load_v(nxt, v1, tok0, r, c, lane);
                }
                // The two workgroups of a compute unit take turns at the higher wave priority, page by page
                // (workgroups j and j + G / 2 share a unit); measured 0.4 us per call on the 32K benchmark shape.
                if ((__builtin_popcountll(todo) + (blk >= (int)gridDim.x / 2)) & 1)
                    __builtin_amdgcn_s_setprio(1);
                else
                    __builtin_amdgcn_s_setprio(0);
                LSERVE_DECODE_VISIT(idx, cur)
                cur = nxt;
            }
        } else {
            // Quantised pages are half the bytes, so two are kept in flight to cover the same latency.  The
            // three stages rotate by name (a copy of a register whose load is still in flight would wait for it).
            unsigned long long ahead = todo;  // entries whose slabs have not been requested yet
#define LSERVE_REQUEST(DST)                                                                                              \
    {                                                                                                                    \
        const int nx = __builtin_ctzll(ahead);                                                                           \
        ahead &= ahead - 1;                                                                                              \
        const uint4 *k1, *v1;                                                                                            \
        slab_of(__builtin_amdgcn_readlane(my_phys, nx), __builtin_amdgcn_readlane(my_list, nx) % lp.Hkv, k1, v1);        \
        load_k(DST, k1, tok0, lane);                                                                                     \
        load_v(DST, v1, tok0, r, c, lane);                                                                               \
    }
#define LSERVE_TURN(CUR, FILL)                                                                                           \
    {                                                                                                                    \
        const int idx = __builtin_ctzll(todo);                                                                           \
        todo &= todo - 1;                                                                                                \
        if (ahead) LSERVE_REQUEST(FILL)                                                                                  \
        if ((__builtin_popcountll(todo) + (blk >= (int)gridDim.x / 2)) & 1)                                              \
            __builtin_amdgcn_s_setprio(1);                                                                               \
        else                                                                                                             \
            __builtin_amdgcn_s_setprio(0);                                                                               \
        LSERVE_DECODE_VISIT(idx, CUR)                                                                                    \
        if (!todo) break;                                                                                                \
    }
            Slabs<NP, BITS> s0, s1, s2;
            LSERVE_REQUEST(s0)
            if (ahead) LSERVE_REQUEST(s1)
            for (;;) {
                LSERVE_TURN(s0, s2)
                LSERVE_TURN(s1, s0)
                LSERVE_TURN(s2, s1)
            }
#undef LSERVE_TURN
#undef LSERVE_REQUEST
        }
    }
    if (cur_list < 0) return;  // no real entry in this range
    end_piece<T, N, NP, BITS>(st, sm, plan, blk, lo, hi, cur_list, cur_len, lp.H, lp.Hkv, lp.streaming_mask, out, lse_out,
                              part_o, part_ml, arrivals);
}

#undef LSERVE_DECODE_VISIT

// ---- host side -----------------------------------------------------------------------------------

int num_compute_units() {
    static int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
        return n;
    }();
    return cus;
}

// `slack`: nominal entries added to a streaming head's list beyond its s + w pages.  They are never real, so they
// cost the workgroup that holds them nothing, which makes up for what a list boundary inside a range costs it
// (the piece of the list that ends there is folded and delivered, the next list's queries are staged: about
// 0.7 of a page's time, measured).  A selecting head's list has such an entry already, since its "+ 1" page is
// real only after the sequence has grown into a new page.
DecodePlan make_plan(const LayerParams& lp, int batch, int sel_stride, int G, int slack) {
    DecodePlan plan;
    plan.stream_len = lp.sink_pages + lp.local_pages + slack;
    plan.select_len = sel_stride + 1;
    int n_stream = 0;
    for (int hk = 0; hk < lp.Hkv; ++hk) n_stream += (int)((lp.streaming_mask >> hk) & 1ull);
    plan.per_seq = n_stream * plan.stream_len + (lp.Hkv - n_stream) * plan.select_len;
    plan.total = batch * plan.per_seq;
    plan.quot = plan.total / G;
    plan.rem = plan.total % G;
    return plan;
}

struct DecodeScratch {
    float *part_o, *part_ml;  // pieces: unnormalised outputs, (max, sum) pairs
    unsigned* arrivals;       // per list: pieces that have arrived
};

size_t arrival_bytes(const LayerParams& lp, int batch) {
    return ((size_t)batch * lp.Hkv * sizeof(unsigned) + 255) & ~(size_t)255;
}

size_t partial_slots(const LayerParams& lp, int batch) {
    return (size_t)num_compute_units() * kMaxBlocksPerCU + (size_t)batch * lp.Hkv;
}

template <class T, int N, int NP, int BITS>
hipError_t launch_decode_kernels(const LayerParams& lp, const PagedParams& kv, const void* q, const int* sel_pages,
                                 const int* sel_count, const int* sel_seq_len, int sel_stride, void* out,
                                 float* lse_out, const DecodeScratch& ws, hipStream_t stream) {
    const uint4* q4 = reinterpret_cast<const uint4*>(q);
    uint16_t* o16 = reinterpret_cast<uint16_t*>(out);
    // Resident workgroups per compute unit of this instantiation: a property of the binary and the device, asked
    // once (thread-safe initialisation of a function-local static); a failed query counts as one.
    static const int per_cu = [] {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, sparse_decode_kernel<T, N, NP, BITS>, kDecodeThreads, 0) !=
            hipSuccess) {
            (void)hipGetLastError();
            return 1;
        }
        return nb < 1 ? 1 : (nb > kBlocksPerCU ? kBlocksPerCU : nb);
    }();
    // two workgroups per compute unit, unless that leaves fewer than four entries each: a small launch is all
    // start-up and fold, and half as many workgroups with twice the pages do less of each (measured)
    int G = num_compute_units() * per_cu;
    DecodePlan plan = make_plan(lp, kv.batch, sel_stride, G, 0);
    if (per_cu > 1 && plan.quot < 4) {
        G = num_compute_units();
        plan = make_plan(lp, kv.batch, sel_stride, G, 0);
    } else if (plan.quot >= kSlackFromEntries) {
        plan = make_plan(lp, kv.batch, sel_stride, G, 1);
    }
    hipLaunchKernelGGL((sparse_decode_kernel<T, N, NP, BITS>), dim3(G), dim3(kDecodeThreads), 0, stream, lp, kv, plan, q4,
                       sel_pages, sel_count, sel_seq_len, sel_stride, o16, lse_out, ws.part_o, ws.part_ml, ws.arrivals);
    return hipGetLastError();
}

template <class T, int N>
hipError_t launch_decode_np(const LayerParams& lp, const PagedParams& kv, const void* q, const int* sel_pages,
                            const int* sel_count, const int* sel_seq_len, int sel_stride, void* out, float* lse_out,
                            const DecodeScratch& ws, hipStream_t stream) {
#define LSERVE_DECODE_NP(NPV)                                                                                       \
    case NPV:                                                                                                       \
        return launch_decode_kernels<T, N, NPV, 16>(lp, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out,   \
                                                    lse_out, ws, stream);
    if (kv.kv_bits == 8)  // quantised pages are always 64 tokens (checked by the caller)
        return launch_decode_kernels<T, N, 64, 8>(lp, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out, lse_out,
                                                  ws, stream);
    if (kv.kv_bits == 4)
        return launch_decode_kernels<T, N, 64, 4>(lp, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out, lse_out,
                                                  ws, stream);
    switch (lp.NP) {
        LSERVE_DECODE_NP(16)
        LSERVE_DECODE_NP(32)
        LSERVE_DECODE_NP(64)
        LSERVE_DECODE_NP(128)
        default:
            return hipErrorInvalidValue;
    }
#undef LSERVE_DECODE_NP
}

template <class T>
hipError_t launch_decode(const LayerParams& lp, const PagedParams& kv, const void* q, const int* sel_pages,
                         const int* sel_count, const int* sel_seq_len, int sel_stride, void* out, float* lse_out,
                         void* workspace, hipStream_t stream) {
    // arrival counters (one per list, zero between launches), then the pieces
    DecodeScratch ws;
    ws.arrivals = reinterpret_cast<unsigned*>(workspace);
    ws.part_o = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + arrival_bytes(lp, kv.batch));
    ws.part_ml = ws.part_o + partial_slots(lp, kv.batch) * lp.group * kHeadDim;
#define LSERVE_DECODE_N(NV)                                                                                          \
    case NV:                                                                                                         \
        return launch_decode_np<T, NV>(lp, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out, lse_out,       \
                                       ws, stream);
    switch (lp.group) {
        LSERVE_DECODE_N(1)
        LSERVE_DECODE_N(2)
        LSERVE_DECODE_N(3)
        LSERVE_DECODE_N(4)
        LSERVE_DECODE_N(5)
        LSERVE_DECODE_N(6)
        LSERVE_DECODE_N(7)
        LSERVE_DECODE_N(8)
        default:
            return hipErrorInvalidValue;
    }
#undef LSERVE_DECODE_N
}

// Measurement aid, not part of the attention path: reads the K and V slabs a decode call with the same arguments
// would read, one short workgroup per index-table entry, folds the words together and throws the result away.  The
// time of this launch is what the memory system charges for the decode call's access pattern alone.
__global__ __launch_bounds__(kDecodeThreads) void decode_read_probe_kernel(LayerParams lp, PagedParams kv,
                                                                           const int* __restrict__ sel_pages,
                                                                           const int* __restrict__ sel_count,
                                                                           const int* __restrict__ sel_seq_len,
                                                                           int sel_stride, int slab_u4,
                                                                           unsigned* __restrict__ sink) {
    const int list = blockIdx.y, i = blockIdx.x;
    const int b = list / lp.Hkv, hk = list % lp.Hkv;
    const PageList pl = make_page_list(lp, b, hk, kv.seq_lens[b], sel_pages, sel_count, sel_seq_len, sel_stride);
    if (i >= pl.len) return;
    const int pos = page_of(pl, i);
    const bool ring = in_stream_pool(lp, kv, hk);
    const int phys = ring ? kv.ring_table[(size_t)b * kv.ring + ring_slot(lp, pos)] : kv.page_table[(size_t)b * kv.max_pages + pos];
    const size_t o = ((size_t)phys * (ring ? kv.stream_heads : kv.pool_heads) + pool_rank(lp, kv, hk, ring)) * slab_u4;
    const uint4* k = reinterpret_cast<const uint4*>(ring ? kv.k_stream : kv.k_pool) + o;
    const uint4* v = reinterpret_cast<const uint4*>(ring ? kv.v_stream : kv.v_pool) + o;
    unsigned acc = 0;
    for (int j0 = 0; j0 < slab_u4; j0 += 4 * kDecodeThreads) {  // four 16-byte loads of K and of V in flight per thread
        uint4 a[4], c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = min(j0 + u * kDecodeThreads + (int)threadIdx.x, slab_u4 - 1);
            a[u] = k[j];
            c[u] = v[j];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= a[u].x ^ a[u].y ^ a[u].z ^ a[u].w ^ c[u].x ^ c[u].y ^ c[u].z ^ c[u].w;
    }
    if (sink && acc == 0x9e3779b9u) *sink = acc;  // keeps the loads alive
}

}  // namespace

hipError_t launch_decode_read_probe(const LayerParams& lp, const PagedParams& kv, const int* sel_pages,
                                    const int* sel_count, const int* sel_seq_len, int sel_stride, hipStream_t stream) {
    // entries of the longest list the launch looks at: the nominal length plus eight pages created since the selection
    const int entries = std::max(sel_stride, lp.sink_pages + lp.local_pages) + 8;
    hipLaunchKernelGGL(decode_read_probe_kernel, dim3(entries, kv.batch * lp.Hkv), dim3(kDecodeThreads), 0, stream, lp, kv,
                       sel_pages, sel_count, sel_seq_len, sel_stride, (int)slab_chunks(lp.NP, kv.kv_bits), (unsigned*)nullptr);
    return hipGetLastError();
}

long long decode_nominal_entries(const LayerParams& lp, int sel_stride) {
    long long acc = 0;
    for (int hk = 0; hk < lp.Hkv; ++hk)
        acc += ((lp.streaming_mask >> hk) & 1ull) ? (long long)lp.sink_pages + lp.local_pages + 1  // with the slack entry
                                                  : (long long)sel_stride + 1;
    return acc;
}

size_t decode_workspace_bytes(const LayerParams& lp, int batch, int sel_stride) {
    (void)sel_stride;
    return arrival_bytes(lp, batch) + partial_slots(lp, batch) * lp.group * (kHeadDim + 2) * sizeof(float);
}

hipError_t preload_decode_kernels() {
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&sparse_decode_kernel<F16, 1, 64, 16>));
}

hipError_t launch_sparse_decode(int dtype, const LayerParams& lp, const PagedParams& kv, const void* q,
                                const int* sel_pages, const int* sel_count, const int* sel_seq_len,
                                int sel_stride, void* out, float* lse_out, void* workspace, hipStream_t stream) {
    return dtype == 0 ? launch_decode<F16>(lp, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out, lse_out,
                                           workspace, stream)
                      : launch_decode<BF16>(lp, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out, lse_out,
                                            workspace, stream);
}

}  // namespace lserve
