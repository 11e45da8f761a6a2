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
    const size_t ph = (size_t)phys * kv.pool_heads + pool_rank(lp, kv, hk, false);  // (page, head) index inside the main pool
    const uint4* slab = reinterpret_cast<const uint4*>(kv.k_pool) + ph * lp.NP * (kHeadDim / 8);

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
        uint4* dst = reinterpret_cast<uint4*>(kv.stats) + ((ph * lp.g + j) * 2) * (kHeadDim / 8);
        // max / min of stored values are stored values: the conversion back is exact
        dst[c] = make_uint4(Elem<T>::pack(vmax[0], vmax[1]), Elem<T>::pack(vmax[2], vmax[3]),
                            Elem<T>::pack(vmax[4], vmax[5]), Elem<T>::pack(vmax[6], vmax[7]));
        dst[kHeadDim / 8 + c] = make_uint4(Elem<T>::pack(vmin[0], vmin[1]), Elem<T>::pack(vmin[2], vmin[3]),
                                           Elem<T>::pack(vmin[4], vmin[5]), Elem<T>::pack(vmin[6], vmin[7]));
    }
}

// Asymmetric quantisation of one token row held by the 16 lanes of a DPP row, eight features per lane
// (Sec. 3.2: scale factor and zero point of a token are stored next to its features), to codes 0 .. LEVELS:
//   zero = fp16(min), scale = fp16((max - zero) / LEVELS), code = clamp(rint((x - zero) / scale), 0, LEVELS),
// every step in IEEE fp32 (true divisions) so that the codes do not depend on the machine.  Yields the
// lane's eight codes and the token's (scale, zero) pair as two fp16 in one word.
template <class T, int LEVELS>
__device__ __forceinline__ void quantize_row(const uint4& x, uint32_t (&c)[8], uint32_t& scale_zero) {
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
    float f[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = Elem<T>::lo(w[i]);
        f[2 * i + 1] = Elem<T>::hi(w[i]);
    }
    float lo = f[0], hi = f[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
        lo = fminf(lo, f[i]);
        hi = fmaxf(hi, f[i]);
    }
    lo = fminf(lo, dpp_f<kDppXor1>(lo));
    hi = fmaxf(hi, dpp_f<kDppXor1>(hi));
    lo = fminf(lo, dpp_f<kDppXor2>(lo));
    hi = fmaxf(hi, dpp_f<kDppXor2>(hi));
    lo = fminf(lo, dpp_f<kDppHalfMirror>(lo));
    hi = fmaxf(hi, dpp_f<kDppHalfMirror>(hi));
    lo = fminf(lo, dpp_f<kDppMirror>(lo));
    hi = fmaxf(hi, dpp_f<kDppMirror>(hi));
    constexpr float kBig = 65504.f;  // largest finite fp16
    const _Float16 zero_h = (_Float16)fminf(fmaxf(lo, -kBig), kBig);
    const float zero = (float)zero_h;
    const _Float16 scale_h = (_Float16)fminf((hi - zero) / (float)LEVELS, kBig);
    const float scale = (float)scale_h;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float t = fminf(fmaxf(__builtin_rintf((f[i] - zero) / scale), 0.f), (float)LEVELS);
        c[i] = scale > 0.f ? (uint32_t)t : 0u;
    }
    const half2_t sz = {scale_h, zero_h};
    scale_zero = __builtin_bit_cast(uint32_t, sz);
}
// One byte per code, features in order.
__device__ __forceinline__ uint2 pack_codes8(const uint32_t (&c)[8]) {
    return make_uint2(c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24), c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24));
}
// Two codes per byte: byte j of the word holds feature j in its low and feature 4 + j in its high half, so
// that masking out either half leaves four codes in the byte lanes the 8-bit path uses.
__device__ __forceinline__ uint32_t pack_codes4(const uint32_t (&c)[8]) {
    return (c[0] | (c[4] << 4)) | ((c[1] | (c[5] << 4)) << 8) | ((c[2] | (c[6] << 4)) << 16) | ((c[3] | (c[7] << 4)) << 24);
}

// KV write-back with the statistics updated in the same pass (Sec. 3.2, Sec. 3.5.2): one workgroup per
// (physical page touched by the new tokens, KV head, sequence), one wavefront per logical page.  New
// rows are copied into both pools with 16-byte accesses; for non-streaming heads the wave folds the
// new keys into max / min rows and, when the logical page already held tokens, combines them with the
// stored rows instead of re-reading the old keys.  BITS = 8 or 4 stores the rows quantised (one byte or half
// a byte per feature, then the page's (scale, zero) pairs); the statistics are still those of the 16-bit
// keys handed in.
template <class T, int BITS>
__global__ __launch_bounds__(kWave* kMaxLogical) void append_kv_kernel(LayerParams lp, PagedParams kv,
                                                                        const uint4* __restrict__ k_new,
                                                                        const uint4* __restrict__ v_new,
                                                                        const int* __restrict__ cu_new,
                                                                        const int* __restrict__ start_pos) {
    const int b = blockIdx.z, hk = blockIdx.y;
    const int j = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int r = lane / 16, c = lane % 16;
    const int s = start_pos[b], src0 = cu_new[b];
    const int e = s + (cu_new[b + 1] - src0);  // new tokens occupy positions [s, e)
    const int p = s / lp.NP + (int)blockIdx.x;
    const int lo = p * lp.NP + j * lp.NL, hi = lo + lp.NL;  // this wave's logical page
    const int t0 = max(lo, s), t1 = min(hi, e);
    if (t0 >= t1) return;
    const bool streaming = (lp.streaming_mask >> hk) & 1ull;
    size_t ph;  // (page, head) index inside the pool that stores this head
    uint4 *kdst, *vdst;
    if (in_stream_pool(lp, kv, hk)) {
        // bounded pool: only sink pages and the pages that are still local once all new tokens are in
        // are stored; a local page lands on the ring slot of the page w positions before it
        if (p >= lp.sink_pages && p < ceil_div(e, lp.NP) - lp.local_pages) return;
        const int phys = kv.ring_table[(size_t)b * kv.ring + ring_slot(lp, p)];
        ph = (size_t)phys * kv.stream_heads + pool_rank(lp, kv, hk, true);
        kdst = reinterpret_cast<uint4*>(const_cast<void*>(kv.k_stream));
        vdst = reinterpret_cast<uint4*>(const_cast<void*>(kv.v_stream));
    } else {
        const int phys = kv.page_table[(size_t)b * kv.max_pages + p];
        ph = (size_t)phys * kv.pool_heads + pool_rank(lp, kv, hk, false);
        kdst = reinterpret_cast<uint4*>(const_cast<void*>(kv.k_pool));
        vdst = reinterpret_cast<uint4*>(const_cast<void*>(kv.v_pool));
    }
    kdst += ph * slab_chunks(lp.NP, BITS);
    vdst += ph * slab_chunks(lp.NP, BITS);

    float vmax[8], vmin[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        vmax[i] = -INFINITY;
        vmin[i] = INFINITY;
    }
    for (int t = t0 + r; t < t1; t += 4) {
        const size_t src = ((size_t)(src0 + t - s) * lp.Hkv + hk) * (kHeadDim / 8) + c;
        const uint4 x = k_new[src];
        const uint4 y = v_new[src];
        const int slot = t - p * lp.NP;
        if (BITS == 16) {
            const size_t dst = (size_t)slot * (kHeadDim / 8) + c;
            kdst[dst] = x;
            vdst[dst] = y;
        } else {
            uint32_t ksz, vsz, kc[8], vc[8];
            quantize_row<T, (1 << BITS) - 1>(x, kc, ksz);
            quantize_row<T, (1 << BITS) - 1>(y, vc, vsz);
            if (BITS == 8) {
                reinterpret_cast<uint2*>(kdst)[(size_t)slot * (kHeadDim / 8) + c] = pack_codes8(kc);
                reinterpret_cast<uint2*>(vdst)[(size_t)slot * (kHeadDim / 8) + c] = pack_codes8(vc);
            } else {
                reinterpret_cast<uint32_t*>(kdst)[(size_t)slot * (kHeadDim / 8) + c] = pack_codes4(kc);
                reinterpret_cast<uint32_t*>(vdst)[(size_t)slot * (kHeadDim / 8) + c] = pack_codes4(vc);
            }
            if (c == 0) {  // the pairs follow the page's code rows
                reinterpret_cast<uint32_t*>(kdst + lp.NP * (kHeadDim * BITS / 128))[slot] = ksz;
                reinterpret_cast<uint32_t*>(vdst + lp.NP * (kHeadDim * BITS / 128))[slot] = vsz;
            }
        }
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = Elem<T>::lo(w[i]), bb = Elem<T>::hi(w[i]);
            vmax[2 * i] = fmaxf(vmax[2 * i], a);
            vmin[2 * i] = fminf(vmin[2 * i], a);
            vmax[2 * i + 1] = fmaxf(vmax[2 * i + 1], bb);
            vmin[2 * i + 1] = fminf(vmin[2 * i + 1], bb);
        }
    }
    if (streaming) return;  // streaming heads are never scored
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        vmax[i] = rows4_max(vmax[i]);
        vmin[i] = rows4_min(vmin[i]);
    }
    if (r == 0) {
        uint4* st = reinterpret_cast<uint4*>(kv.stats) + ((ph * lp.g + j) * 2) * (kHeadDim / 8);
        if (lo < s) {  // the logical page already held tokens: fold the stored rows in
            const uint4 om = st[c], on = st[kHeadDim / 8 + c];
            const uint32_t wm[4] = {om.x, om.y, om.z, om.w}, wn[4] = {on.x, on.y, on.z, on.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                vmax[2 * i] = fmaxf(vmax[2 * i], Elem<T>::lo(wm[i]));
                vmax[2 * i + 1] = fmaxf(vmax[2 * i + 1], Elem<T>::hi(wm[i]));
                vmin[2 * i] = fminf(vmin[2 * i], Elem<T>::lo(wn[i]));
                vmin[2 * i + 1] = fminf(vmin[2 * i + 1], Elem<T>::hi(wn[i]));
            }
        }
        st[c] = make_uint4(Elem<T>::pack(vmax[0], vmax[1]), Elem<T>::pack(vmax[2], vmax[3]),
                           Elem<T>::pack(vmax[4], vmax[5]), Elem<T>::pack(vmax[6], vmax[7]));
        st[kHeadDim / 8 + c] = make_uint4(Elem<T>::pack(vmin[0], vmin[1]), Elem<T>::pack(vmin[2], vmin[3]),
                                          Elem<T>::pack(vmin[4], vmin[5]), Elem<T>::pack(vmin[6], vmin[7]));
    }
}

hipError_t launch_append_kv(int dtype, const LayerParams& lp, const PagedParams& kv, const void* k_new, const void* v_new,
                            const int* cu_new, const int* start_pos, int max_new_per_seq, hipStream_t stream) {
    // the new tokens of a sequence touch at most ceil(n / N_P) + 1 physical pages
    dim3 grid((max_new_per_seq + lp.NP - 1) / lp.NP + 1, lp.Hkv, kv.batch);
    dim3 block(kWave * lp.g);
    const uint4* k4 = reinterpret_cast<const uint4*>(k_new);
    const uint4* v4 = reinterpret_cast<const uint4*>(v_new);
    if (kv.kv_bits == 8) {
        if (dtype == 0)
            hipLaunchKernelGGL((append_kv_kernel<F16, 8>), grid, block, 0, stream, lp, kv, k4, v4, cu_new, start_pos);
        else
            hipLaunchKernelGGL((append_kv_kernel<BF16, 8>), grid, block, 0, stream, lp, kv, k4, v4, cu_new, start_pos);
    } else if (kv.kv_bits == 4) {
        if (dtype == 0)
            hipLaunchKernelGGL((append_kv_kernel<F16, 4>), grid, block, 0, stream, lp, kv, k4, v4, cu_new, start_pos);
        else
            hipLaunchKernelGGL((append_kv_kernel<BF16, 4>), grid, block, 0, stream, lp, kv, k4, v4, cu_new, start_pos);
    } else if (dtype == 0) {
        hipLaunchKernelGGL((append_kv_kernel<F16, 16>), grid, block, 0, stream, lp, kv, k4, v4, cu_new, start_pos);
    } else {
        hipLaunchKernelGGL((append_kv_kernel<BF16, 16>), grid, block, 0, stream, lp, kv, k4, v4, cu_new, start_pos);
    }
    return hipGetLastError();
}

hipError_t preload_stats_kernels() {
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&page_stats_kernel<F16>));
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
