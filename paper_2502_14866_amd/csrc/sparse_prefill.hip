// Block-sparse causal prefill attention (Sec. 3.1, Sec. 3.4) on the gfx950 matrix cores.
//
// Mask tiles are 64 x 64 (query tile x key tile = page).  Dense heads visit every key tile up to
// the diagonal; streaming heads visit only the sink tiles and the local band, so whole tiles
// outside the mask are never loaded.  Only the diagonal tile needs element-wise causal masking.
//
// Mapping to CDNA4: a workgroup of four wavefronts owns 256 consecutive query rows of one head;
// wavefront w owns mask tile 4 * block + w (64 rows).  Key tiles are staged through LDS once per
// workgroup and consumed by all four wavefronts.  Scores are computed transposed,
//   S^T (keys x queries) = K (keys x d) * Q^T (d x queries)          v_mfma_f32_32x32x16
// so that a lane owns one query column: the softmax reductions over keys stay inside the lane
// (plus one exchange between the two lane halves), and the exponentiated tile is already in the
// register layout of the B operand of the second product
//   O^T (d x queries) += V^T (d x keys) * P^T (keys x queries).
// V^T tiles come from a small pre-pass that transposes V once per call into 64-key tiles whose key
// order matches the accumulator layout, so every LDS operand read is one 16-byte access.
#include "kernels.h"

namespace lserve {

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf168_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 64;              // mask tile = key tile = page
constexpr int kPrefillThreads = 256;   // 4 waves
constexpr int kRowsPerBlock = 256;     // 4 mask tiles of queries
constexpr int kKRowBytes = 256 + 16;   // K tile row (128 x 16 bit) padded against LDS bank conflicts
constexpr int kVRowBytes = 128 + 16;   // V^T tile row (64 keys x 16 bit) padded
constexpr int kKTileBytes = kTile * kKRowBytes;
constexpr int kVTileBytes = kHeadDim * kVRowBytes;
constexpr float kLn2 = 0.6931471805599453f;

template <class T> struct Mfma;
template <> struct Mfma<F16> {
    static __device__ __forceinline__ float16_t run(uint4 a, uint4 b, float16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<BF16> {
    static __device__ __forceinline__ float16_t run(uint4 a, uint4 b, float16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf168_t, a), __builtin_bit_cast(bf168_t, b), c, 0, 0, 0);
    }
};

// First V^T tile slot of sequence b: floor(cu[b] / 64) + b leaves room for every ragged last tile.
__device__ __forceinline__ int tile_base(int cu_b, int b) { return cu_b / kTile + b; }

// Slot of key (relative to its 64-key tile) inside a V^T tile row.  Register v of a 32 x 32
// accumulator holds row 8 * (v / 4) + 4 * half + v % 4; the second product consumes registers
// 8j .. 8j+7 of each half as one operand, so those eight keys must be contiguous.
__device__ __forceinline__ int vt_slot(int key) {
    const int kb = key / 32, k32 = key % 32;
    const int v = (k32 / 8) * 4 + (k32 % 4), half = (k32 / 4) % 2;
    return kb * 32 + (v / 8) * 16 + half * 8 + (v % 8);
}

// V [total][Hkv][D]  ->  vt [Hkv][tile slot][D][64 key slots]; keys past the sequence end become 0.
template <class T>
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint16_t* __restrict__ v, uint16_t* __restrict__ vt,
                                                          const int* __restrict__ cu_seqlens, int Hkv,
                                                          int tiles_total) {
    __shared__ uint16_t sm[kTile][kHeadDim + 2];
    const int b = blockIdx.z, hk = blockIdx.y, jt = blockIdx.x;
    const int start = cu_seqlens[b], len = cu_seqlens[b + 1] - start;
    if (jt * kTile >= len) return;
    for (int idx = threadIdx.x; idx < kTile * kHeadDim; idx += 256) {
        const int key = idx / kHeadDim, d = idx % kHeadDim;
        const int t = jt * kTile + key;
        sm[key][d] = t < len ? v[((size_t)(start + t) * Hkv + hk) * kHeadDim + d] : (uint16_t)0;
    }
    __syncthreads();
    uint16_t* dst = vt + ((size_t)hk * tiles_total + tile_base(start, b) + jt) * kHeadDim * kTile;
    for (int idx = threadIdx.x; idx < kTile * kHeadDim; idx += 256) {
        const int d = idx / kTile, key = idx % kTile;
        dst[(size_t)d * kTile + vt_slot(key)] = sm[key][d];
    }
}

template <class T>
__device__ __forceinline__ uint4 pack8(const float* p) {
    return make_uint4(Elem<T>::pack(p[0], p[1]), Elem<T>::pack(p[2], p[3]), Elem<T>::pack(p[4], p[5]),
                      Elem<T>::pack(p[6], p[7]));
}

template <class T>
__global__ __launch_bounds__(kPrefillThreads) void sparse_prefill_kernel(
    LayerParams lp, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ vt,
    const int* __restrict__ cu_seqlens, int batch, int blocks_per_seq, int tiles_total, uint16_t* __restrict__ out,
    float* __restrict__ lse_out, int total_tokens) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // two stages of (K tile, V^T tile)
    constexpr int kStageBytes = kKTileBytes + kVTileBytes;

    // heaviest query blocks first; heads of one GQA group are neighbours
    const int h = blockIdx.x % lp.H;
    const int rest = blockIdx.x / lp.H;
    const int b = rest % batch;
    const int qblk = blocks_per_seq - 1 - rest / batch;
    const int hk = h / lp.group;
    const int start = cu_seqlens[b], len = cu_seqlens[b + 1] - start;
    if (qblk * kRowsPerBlock >= len) return;

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int n = lane % 32, half = lane / 32;
    const bool streaming = (lp.streaming_mask >> hk) & 1ull;
    const int iq = qblk * 4 + wave;               // this wave's mask tile
    const int n_qtiles = ceil_div(len, kTile);
    const int iq_last = min(qblk * 4 + 3, n_qtiles - 1);  // last mask tile of the block that holds rows
    const bool wave_has_rows = iq < n_qtiles;

    // key tiles the block visits: [0, sink_end) and [band_begin, iq_last]
    int sink_end, band_begin;
    if (streaming) {
        band_begin = max(0, qblk * 4 - lp.local_pages + 1);
        sink_end = min(lp.sink_pages, band_begin);
    } else {
        band_begin = 0;
        sink_end = 0;
    }
    const int n_visit = sink_end + (iq_last - band_begin + 1);

    // ---- Q^T operands: lane (n, half) holds Q[row][16 kk + 8 half .. + 8] for both 32-row blocks
    uint4 qreg[2][8];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int row = min(iq * kTile + qb * 32 + n, len - 1);
        const uint4* src = reinterpret_cast<const uint4*>(q + ((size_t)(start + row) * lp.H + h) * kHeadDim);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qreg[qb][kk] = src[kk * 2 + half];
    }

    float16_t acc[4][2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[db][qb][i] = 0.f;
    float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.f, 0.f};

    // ---- staging: each thread moves 4 x 16 B of the K tile and 4 x 16 B of the V^T tile
    const uint16_t* kbase = k + ((size_t)start * lp.Hkv + hk) * kHeadDim;
    const uint16_t* vtbase = vt + ((size_t)hk * tiles_total + tile_base(start, b)) * kHeadDim * kTile;
    uint4 kst[4], vst[4];
    auto tile_of = [&](int it) { return it < sink_end ? it : band_begin + (it - sink_end); };
    auto fetch = [&](int jt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int chunk = tid + i * kPrefillThreads;  // 1024 chunks of 16 B per tile
            const int krow = min(jt * kTile + chunk / 16, len - 1);
            kst[i] = reinterpret_cast<const uint4*>(kbase + (size_t)krow * lp.Hkv * kHeadDim)[chunk % 16];
            vst[i] = reinterpret_cast<const uint4*>(vtbase + (size_t)jt * kHeadDim * kTile)[chunk];
        }
    };
    auto stash = [&](int stage) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int chunk = tid + i * kPrefillThreads;
            *reinterpret_cast<uint4*>(smem + stage * kStageBytes + (chunk / 16) * kKRowBytes + (chunk % 16) * 16) = kst[i];
            *reinterpret_cast<uint4*>(smem + stage * kStageBytes + kKTileBytes + (chunk / 8) * kVRowBytes + (chunk % 8) * 16) = vst[i];
        }
    };

    fetch(tile_of(0));
    stash(0);
    __syncthreads();

    for (int it = 0; it < n_visit; ++it) {
        const int stage = it & 1;
        const int jt = tile_of(it);
        if (it + 1 < n_visit) fetch(tile_of(it + 1));

        // does this wave's mask tile keep key tile jt?
        bool keep = wave_has_rows && jt <= iq;
        if (streaming) keep = keep && (jt < lp.sink_pages || jt > iq - lp.local_pages);
        if (keep) {
            const unsigned char* ks = smem + stage * kStageBytes;
            const unsigned char* vs = ks + kKTileBytes;
            // S^T for the 64 keys of the tile: [key block][query block]
            float16_t s[2][2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[kb][qb][i] = 0.f;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const uint4 a = *reinterpret_cast<const uint4*>(ks + (kb * 32 + n) * kKRowBytes + kk * 32 + half * 16);
                    s[kb][0] = Mfma<T>::run(a, qreg[0][kk], s[kb][0]);
                    s[kb][1] = Mfma<T>::run(a, qreg[1][kk], s[kb][1]);
                }
            }
            const bool diagonal = jt == iq;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                float mx = -INFINITY;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float x = s[kb][qb][i] * lp.sm_scale_log2;
                        if (diagonal) {
                            const int key = kb * 32 + 8 * (i / 4) + 4 * half + (i % 4);
                            if (key > qb * 32 + n) x = -INFINITY;
                        }
                        s[kb][qb][i] = x;
                        mx = fmaxf(mx, x);
                    }
                }
                mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
                const float m_new = fmaxf(m[qb], mx);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f(m[qb] - m_safe);
                m[qb] = m_new;
                float ps = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float p = __builtin_amdgcn_exp2f(s[kb][qb][i] - m_safe);
                        s[kb][qb][i] = p;
                        ps += p;
                    }
                l[qb] = l[qb] * alpha + ps;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[db][qb][i] *= alpha;
            }
            // O^T += V^T * P^T, 16 keys per instruction
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    float pf0[8], pf1[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        pf0[e] = s[kb][0][8 * j + e];
                        pf1[e] = s[kb][1][8 * j + e];
                    }
                    const uint4 p0 = pack8<T>(pf0), p1 = pack8<T>(pf1);
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const uint4 a = *reinterpret_cast<const uint4*>(vs + (db * 32 + n) * kVRowBytes +
                                                                        (kb * 32 + j * 16 + half * 8) * 2);
                        acc[db][0] = Mfma<T>::run(a, p0, acc[db][0]);
                        acc[db][1] = Mfma<T>::run(a, p1, acc[db][1]);
                    }
                }
            }
        }
        if (it + 1 < n_visit) stash(stage ^ 1);
        __syncthreads();
    }

    if (!wave_has_rows) return;
    // ---- epilogue: lane (n, half) holds O^T[d][q] for d = 32 db + 8 (i / 4) + 4 half + i % 4
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float lt = l[qb] + __shfl_xor(l[qb], 32, kWave);
        const int row = iq * kTile + qb * 32 + n;
        if (row >= len) continue;
        const float inv = 1.f / lt;
        uint16_t* dst = out + ((size_t)(start + row) * lp.H + h) * kHeadDim;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int d = db * 32 + 8 * g4 + 4 * half;
                uint2 w;
                w.x = Elem<T>::pack(acc[db][qb][4 * g4] * inv, acc[db][qb][4 * g4 + 1] * inv);
                w.y = Elem<T>::pack(acc[db][qb][4 * g4 + 2] * inv, acc[db][qb][4 * g4 + 3] * inv);
                *reinterpret_cast<uint2*>(dst + d) = w;
            }
        if (lse_out && half == 0)
            lse_out[(size_t)h * total_tokens + start + row] = (m[qb] + __builtin_amdgcn_logf(lt)) * kLn2;
    }
}

int prefill_tile_slots(int total_tokens, int batch) { return total_tokens / kTile + batch; }

template <class T>
hipError_t launch_prefill(const LayerParams& lp, const void* q, const void* k, const void* v, const int* cu_seqlens,
                          int batch, int total_tokens, int max_seqlen, void* out, float* lse_out, void* workspace,
                          hipStream_t stream) {
    const int tiles_total = prefill_tile_slots(total_tokens, batch);
    uint16_t* vt = reinterpret_cast<uint16_t*>(workspace);
    const int max_tiles = (max_seqlen + kTile - 1) / kTile;
    hipLaunchKernelGGL(transpose_v_kernel<T>, dim3(max_tiles, lp.Hkv, batch), dim3(256), 0, stream,
                       reinterpret_cast<const uint16_t*>(v), vt, cu_seqlens, lp.Hkv, tiles_total);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int blocks_per_seq = (max_seqlen + kRowsPerBlock - 1) / kRowsPerBlock;
    const size_t lds = 2 * (size_t)(kKTileBytes + kVTileBytes);
    static bool attr_done = false;  // one flag per element type (this function is a template)
    if (!attr_done) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sparse_prefill_kernel<T>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(sparse_prefill_kernel<T>, dim3(blocks_per_seq * batch * lp.H), dim3(kPrefillThreads), lds, stream,
                       lp, reinterpret_cast<const uint16_t*>(q), reinterpret_cast<const uint16_t*>(k), vt, cu_seqlens,
                       batch, blocks_per_seq, tiles_total, reinterpret_cast<uint16_t*>(out), lse_out, total_tokens);
    return hipGetLastError();
}

}  // namespace

size_t prefill_workspace_bytes(const LayerParams& lp, int total_tokens, int batch) {
    return (size_t)lp.Hkv * prefill_tile_slots(total_tokens, batch) * kHeadDim * kTile * sizeof(uint16_t);
}

hipError_t launch_sparse_prefill(int dtype, const LayerParams& lp, const void* q, const void* k, const void* v,
                                 const int* cu_seqlens, int batch, int total_tokens, int max_seqlen, void* out,
                                 float* lse_out, void* workspace, hipStream_t stream) {
    return dtype == 0 ? launch_prefill<F16>(lp, q, k, v, cu_seqlens, batch, total_tokens, max_seqlen, out, lse_out,
                                            workspace, stream)
                      : launch_prefill<BF16>(lp, q, k, v, cu_seqlens, batch, total_tokens, max_seqlen, out, lse_out,
                                             workspace, stream);
}

}  // namespace lserve
