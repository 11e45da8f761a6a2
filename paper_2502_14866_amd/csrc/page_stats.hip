// Key statistics for hierarchical paging (Sec. 3.5.2): channel-wise max / min of the keys of
// every logical page of the non-streaming KV heads.  Pure streaming work: one wavefront reads one
// logical page with 16-byte loads (16 lanes cover one 256-byte token row, the four rows of the
// wave cover four tokens per load) and folds the rows together at the end.
#include "kernels.h"

namespace lserve {

template <class T>
__global__ __launch_bounds__(kWave* kMaxLogical) void page_stats_kernel(LayerParams lp, PagedParams kv,
                                                                         const int* __restrict__ start_pos,
                                                                         HeadList heads) {
    const int b = blockIdx.z;
    const int hk = heads.idx[blockIdx.y];
    const int j = threadIdx.x / kWave;  // logical page inside the physical page
    const int lane = threadIdx.x % kWave;
    const int L = kv.seq_lens[b];
    const int start = start_pos ? start_pos[b] : 0;
    const int P = ceil_div(L, lp.NP);
    const int p = P - 1 - (int)blockIdx.x;  // pages are visited from the tail
    if (p < 0 || p < start / lp.NP) return;
    const int lo = p * lp.NP + j * lp.NL;
    const int hi = min(lo + lp.NL, L);
    if (lo >= L || hi <= start) return;

    const int phys = kv.page_table[(size_t)b * kv.max_pages + p];
    const int r = lane / 16, c = lane % 16;
    const uint4* slab = reinterpret_cast<const uint4*>(kv.k_pool) + ((size_t)phys * lp.Hkv + hk) * lp.NP * (kHeadDim / 8);

    float vmax[8], vmin[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        vmax[i] = -INFINITY;
        vmin[i] = INFINITY;
    }
    for (int t = lo + r; t < hi; t += 4) {
        uint4 x = slab[(size_t)(t - p * lp.NP) * (kHeadDim / 8) + c];
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float a = Elem<T>::lo(w[i]), bb = Elem<T>::hi(w[i]);
            vmax[2 * i] = fmaxf(vmax[2 * i], a);
            vmin[2 * i] = fminf(vmin[2 * i], a);
            vmax[2 * i + 1] = fmaxf(vmax[2 * i + 1], bb);
            vmin[2 * i + 1] = fminf(vmin[2 * i + 1], bb);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        vmax[i] = rows4_max(vmax[i]);
        vmin[i] = rows4_min(vmin[i]);
    }
    if (r == 0) {
        uint4* dst = reinterpret_cast<uint4*>(kv.stats) + ((((size_t)phys * lp.Hkv + hk) * lp.g + j) * 2) * (kHeadDim / 8);
        // max / min of stored values are stored values: the conversion back is exact
        dst[c] = make_uint4(Elem<T>::pack(vmax[0], vmax[1]), Elem<T>::pack(vmax[2], vmax[3]),
                            Elem<T>::pack(vmax[4], vmax[5]), Elem<T>::pack(vmax[6], vmax[7]));
        dst[kHeadDim / 8 + c] = make_uint4(Elem<T>::pack(vmin[0], vmin[1]), Elem<T>::pack(vmin[2], vmin[3]),
                                           Elem<T>::pack(vmin[4], vmin[5]), Elem<T>::pack(vmin[6], vmin[7]));
    }
}

hipError_t launch_page_stats(int dtype, const LayerParams& lp, const PagedParams& kv, const int* start_pos,
                             int tail_pages, const HeadList& heads, hipStream_t stream) {
    if (heads.count == 0) return hipSuccess;
    dim3 grid(tail_pages, heads.count, kv.batch);
    dim3 block(kWave * lp.g);
    if (dtype == 0)
        hipLaunchKernelGGL(page_stats_kernel<F16>, grid, block, 0, stream, lp, kv, start_pos, heads);
    else
        hipLaunchKernelGGL(page_stats_kernel<BF16>, grid, block, 0, stream, lp, kv, start_pos, heads);
    return hipGetLastError();
}

}  // namespace lserve
