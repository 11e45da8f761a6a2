// Paged sparse decode attention (Sec. 3.6): one query token per sequence attends only the pages of
// its index table -- the selector's list (plus pages newer than the selection) for dense heads,
// sink + local pages for streaming heads.  Both kinds run in one launch.
//
// The work is GEMV-shaped (n <= 8 query rows per KV head) and bound by HBM bandwidth, so there is
// no MFMA here: each page is a 2 * N_P * 256-byte contiguous K / V slab read with 16-byte loads
// (16 lanes per token row), dot products use packed 16-bit dot instructions with fp32
// accumulation, and the softmax is kept online per wavefront.
//
// Decomposition: the page list of one (sequence, KV head) is cut into chunks; one workgroup of
// four wavefronts walks a chunk page by page, each wavefront taking a quarter of the page's
// tokens, and prefetches the next page's slabs while it works on the current one.  A chunk's
// result is either final (single chunk) or a partial (max, sum, unnormalised output) that a small
// merge kernel combines in chunk order, which keeps the result deterministic.
#include "kernels.h"

namespace lserve {

namespace {

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = kDecodeThreads / kWave;
constexpr int kChunkPages = 8;  // target pages per workgroup
constexpr float kLn2 = 0.6931471805599453f;

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

__device__ __forceinline__ int active_chunks(int len, int slots) { return min(slots, ceil_div(len, kChunkPages)); }

template <int ITS> struct Slabs {
    uint4 k[ITS], v[ITS];
};

template <int ITS>
__device__ __forceinline__ void load_slabs(Slabs<ITS>& s, const uint4* kslab, const uint4* vslab, int tok0, int r, int c) {
#pragma unroll
    for (int it = 0; it < ITS; ++it) s.k[it] = kslab[(size_t)(tok0 + 4 * it + r) * (kHeadDim / 8) + c];
#pragma unroll
    for (int it = 0; it < ITS; ++it) s.v[it] = vslab[(size_t)(tok0 + 4 * it + r) * (kHeadDim / 8) + c];
}

template <class T, int N, int NP>
__global__ __launch_bounds__(kDecodeThreads) void sparse_decode_kernel(
    LayerParams lp, PagedParams kv, const uint4* __restrict__ q, const int* __restrict__ sel_pages,
    const int* __restrict__ sel_count, const int* __restrict__ sel_seq_len, int sel_stride,
    uint16_t* __restrict__ out, float* __restrict__ lse_out, float* __restrict__ part_o, float* __restrict__ part_ml) {
    constexpr int ITS = NP / 16;  // 16-byte loads per lane and slab: the wave covers NP / 4 tokens
    __shared__ float sm_o[kDecodeWaves][N][kHeadDim];
    __shared__ float sm_m[kDecodeWaves][N], sm_l[kDecodeWaves][N];

    const int slot = blockIdx.x, slots = gridDim.x, hk = blockIdx.y, b = blockIdx.z;
    const int L = kv.seq_lens[b];
    const PageList pl = make_page_list(lp, b, hk, L, sel_pages, sel_count, sel_seq_len, sel_stride);
    const int A = active_chunks(pl.len, slots);
    if (slot >= A) return;
    const int i0 = (int)((long long)slot * pl.len / A), i1 = (int)((long long)(slot + 1) * pl.len / A);

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int r = lane / 16, c = lane % 16;
    const int tok0 = wave * (NP / 4);

    uint32_t qreg[N][4];
#pragma unroll
    for (int hh = 0; hh < N; ++hh) {
        uint4 x = q[((size_t)b * lp.H + hk * N + hh) * (kHeadDim / 8) + c];
        qreg[hh][0] = x.x;
        qreg[hh][1] = x.y;
        qreg[hh][2] = x.z;
        qreg[hh][3] = x.w;
    }

    float m[N], l[N], o[N][8];
#pragma unroll
    for (int hh = 0; hh < N; ++hh) {
        m[hh] = -INFINITY;
        l[hh] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[hh][i] = 0.f;
    }

    const uint4* kpool = reinterpret_cast<const uint4*>(kv.k_pool);
    const uint4* vpool = reinterpret_cast<const uint4*>(kv.v_pool);
    const size_t slab = (size_t)NP * (kHeadDim / 8);  // uint4 per (page, head)

    for (int base = i0; base < i1; base += kWave) {
        // every lane fetches the table entries of one list item; they are broadcast page by page
        const int cnt = min(kWave, i1 - base);
        int my_pos = 0, my_phys = 0;
        if (lane < cnt) {
            my_pos = page_of(pl, base + lane);
            my_phys = kv.page_table[(size_t)b * kv.max_pages + my_pos];
        }
        Slabs<ITS> cur, nxt;
        {
            const int phys = __builtin_amdgcn_readfirstlane(my_phys);
            const size_t off = ((size_t)phys * lp.Hkv + hk) * slab;
            load_slabs<ITS>(cur, kpool + off, vpool + off, tok0, r, c);
        }
        for (int idx = 0; idx < cnt; ++idx) {
            if (idx + 1 < cnt) {
                const int phys = __builtin_amdgcn_readlane(my_phys, idx + 1);
                const size_t off = ((size_t)phys * lp.Hkv + hk) * slab;
                load_slabs<ITS>(nxt, kpool + off, vpool + off, tok0, r, c);
            }
            const int pos = __builtin_amdgcn_readlane(my_pos, idx);
            const int valid = L - pos * NP;  // tokens of this page below the sequence length (may exceed NP)

            float s[ITS][N];
#pragma unroll
            for (int it = 0; it < ITS; ++it) {
                const uint32_t kw[4] = {cur.k[it].x, cur.k[it].y, cur.k[it].z, cur.k[it].w};
#pragma unroll
                for (int hh = 0; hh < N; ++hh) {
                    float a = 0.f;
#pragma unroll
                    for (int i = 0; i < 4; ++i) a = Elem<T>::dot2(qreg[hh][i], kw[i], a);
                    s[it][hh] = row16_sum(a) * lp.sm_scale_log2;
                }
            }
            if (valid < NP) {  // tail page: mask the slots past the sequence end, keys and values
#pragma unroll
                for (int it = 0; it < ITS; ++it) {
                    if (tok0 + 4 * it + r >= valid) {
#pragma unroll
                        for (int hh = 0; hh < N; ++hh) s[it][hh] = -INFINITY;
                        cur.v[it] = make_uint4(0, 0, 0, 0);
                    }
                }
            }
            float p[ITS][N];
#pragma unroll
            for (int hh = 0; hh < N; ++hh) {
                float pm = s[0][hh];
#pragma unroll
                for (int it = 1; it < ITS; ++it) pm = fmaxf(pm, s[it][hh]);
                pm = rows4_max(pm);
                const float m_new = fmaxf(m[hh], pm);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f(m[hh] - m_safe);
                m[hh] = m_new;
                float ps = 0.f;
#pragma unroll
                for (int it = 0; it < ITS; ++it) {
                    p[it][hh] = __builtin_amdgcn_exp2f(s[it][hh] - m_safe);
                    ps += p[it][hh];
                }
                l[hh] = l[hh] * alpha + ps;
#pragma unroll
                for (int i = 0; i < 8; ++i) o[hh][i] *= alpha;
            }
#pragma unroll
            for (int it = 0; it < ITS; ++it) {
                const uint32_t vw[4] = {cur.v[it].x, cur.v[it].y, cur.v[it].z, cur.v[it].w};
#pragma unroll
                for (int hh = 0; hh < N; ++hh) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        o[hh][2 * i] = __builtin_fmaf(p[it][hh], Elem<T>::lo(vw[i]), o[hh][2 * i]);
                        o[hh][2 * i + 1] = __builtin_fmaf(p[it][hh], Elem<T>::hi(vw[i]), o[hh][2 * i + 1]);
                    }
                }
            }
            cur = nxt;
        }
    }

    // fold the four token rows of the wave, then the four waves of the workgroup
#pragma unroll
    for (int hh = 0; hh < N; ++hh) {
        l[hh] = rows4_sum(l[hh]);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[hh][i] = rows4_sum(o[hh][i]);
        if (r == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) sm_o[wave][hh][8 * c + i] = o[hh][i];
        }
        if (lane == 0) {
            sm_m[wave][hh] = m[hh];
            sm_l[wave][hh] = l[hh];
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < N * kHeadDim; idx += kDecodeThreads) {
        const int hh = idx / kHeadDim, ch = idx % kHeadDim;
        float M = sm_m[0][hh];
#pragma unroll
        for (int w = 1; w < kDecodeWaves; ++w) M = fmaxf(M, sm_m[w][hh]);
        float lt = 0.f, acc = 0.f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            const float f = __builtin_amdgcn_exp2f(sm_m[w][hh] - M);
            lt += sm_l[w][hh] * f;
            acc += sm_o[w][hh][ch] * f;
        }
        const int h = hk * N + hh;
        if (A == 1) {
            out[((size_t)b * lp.H + h) * kHeadDim + ch] = (uint16_t)(Elem<T>::pack(acc / lt, 0.f) & 0xffffu);
            if (lse_out && ch == 0) lse_out[b * lp.H + h] = (M + __builtin_amdgcn_logf(lt)) * kLn2;
        } else {
            const size_t pi = ((size_t)b * lp.H + h) * slots + slot;
            part_o[pi * kHeadDim + ch] = acc;
            if (ch == 0) {
                part_ml[pi * 2] = M;
                part_ml[pi * 2 + 1] = lt;
            }
        }
    }
}

// Combines the partial results of one (sequence, query head) in chunk order.
template <class T>
__global__ __launch_bounds__(kHeadDim) void decode_merge_kernel(LayerParams lp, PagedParams kv,
                                                                const int* __restrict__ sel_pages,
                                                                const int* __restrict__ sel_count,
                                                                const int* __restrict__ sel_seq_len, int sel_stride,
                                                                int slots, uint16_t* __restrict__ out,
                                                                float* __restrict__ lse_out,
                                                                const float* __restrict__ part_o,
                                                                const float* __restrict__ part_ml) {
    const int h = blockIdx.x, b = blockIdx.y, ch = threadIdx.x;
    const int hk = h / lp.group;
    const PageList pl = make_page_list(lp, b, hk, kv.seq_lens[b], sel_pages, sel_count, sel_seq_len, sel_stride);
    const int A = active_chunks(pl.len, slots);
    if (A <= 1) return;  // the decode kernel already wrote the final result
    const size_t p0 = ((size_t)b * lp.H + h) * slots;
    float M = -INFINITY;
    for (int cI = 0; cI < A; ++cI) M = fmaxf(M, part_ml[(p0 + cI) * 2]);
    float lt = 0.f, acc = 0.f;
    for (int cI = 0; cI < A; ++cI) {
        const float f = __builtin_amdgcn_exp2f(part_ml[(p0 + cI) * 2] - M);
        lt += part_ml[(p0 + cI) * 2 + 1] * f;
        acc += part_o[(p0 + cI) * kHeadDim + ch] * f;
    }
    out[((size_t)b * lp.H + h) * kHeadDim + ch] = (uint16_t)(Elem<T>::pack(acc / lt, 0.f) & 0xffffu);
    if (lse_out && ch == 0) lse_out[b * lp.H + h] = (M + __builtin_amdgcn_logf(lt)) * kLn2;
}

int decode_slots(const LayerParams& lp, int sel_stride) {
    int longest = 0;
    for (int hk = 0; hk < lp.Hkv; ++hk) {
        const bool streaming = (lp.streaming_mask >> hk) & 1ull;
        // dense heads: the selection plus one page created since; longer lists only make chunks longer
        const int len = streaming ? lp.sink_pages + lp.local_pages : sel_stride + 1;
        longest = len > longest ? len : longest;
    }
    const int slots = (longest + kChunkPages - 1) / kChunkPages;
    return slots < 1 ? 1 : slots;
}

template <class T, int N>
hipError_t launch_decode_np(const LayerParams& lp, const PagedParams& kv, const void* q, const int* sel_pages,
                            const int* sel_count, const int* sel_seq_len, int sel_stride, void* out,
                            float* lse_out, float* part_o, float* part_ml, int slots, hipStream_t stream) {
    dim3 grid(slots, lp.Hkv, kv.batch), block(kDecodeThreads);
    const uint4* q4 = reinterpret_cast<const uint4*>(q);
    uint16_t* o16 = reinterpret_cast<uint16_t*>(out);
#define LSERVE_DECODE_NP(NPV)                                                                                  \
    case NPV:                                                                                                  \
        hipLaunchKernelGGL((sparse_decode_kernel<T, N, NPV>), grid, block, 0, stream, lp, kv, q4, sel_pages,   \
                           sel_count, sel_seq_len, sel_stride, o16, lse_out, part_o, part_ml);                 \
        break;
    switch (lp.NP) {
        LSERVE_DECODE_NP(16)
        LSERVE_DECODE_NP(32)
        LSERVE_DECODE_NP(64)
        LSERVE_DECODE_NP(128)
        default:
            return hipErrorInvalidValue;
    }
#undef LSERVE_DECODE_NP
    return hipGetLastError();
}

template <class T>
hipError_t launch_decode(const LayerParams& lp, const PagedParams& kv, const void* q, const int* sel_pages,
                         const int* sel_count, const int* sel_seq_len, int sel_stride, void* out, float* lse_out,
                         void* workspace, hipStream_t stream) {
    const int slots = decode_slots(lp, sel_stride);
    float* part_o = reinterpret_cast<float*>(workspace);
    float* part_ml = part_o + (size_t)kv.batch * lp.H * slots * kHeadDim;
    hipError_t e;
#define LSERVE_DECODE_N(NV)                                                                                         \
    case NV:                                                                                                        \
        e = launch_decode_np<T, NV>(lp, kv, q, sel_pages, sel_count, sel_seq_len, sel_stride, out, lse_out, part_o, \
                                    part_ml, slots, stream);                                                        \
        break;
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
    if (e != hipSuccess) return e;
    if (slots > 1) {
        hipLaunchKernelGGL(decode_merge_kernel<T>, dim3(lp.H, kv.batch), dim3(kHeadDim), 0, stream, lp, kv, sel_pages,
                           sel_count, sel_seq_len, sel_stride, slots, reinterpret_cast<uint16_t*>(out), lse_out,
                           part_o, part_ml);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace

size_t decode_workspace_bytes(const LayerParams& lp, int batch, int sel_stride) {
    const int slots = decode_slots(lp, sel_stride);
    return (size_t)batch * lp.H * slots * (kHeadDim + 2) * sizeof(float);
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
