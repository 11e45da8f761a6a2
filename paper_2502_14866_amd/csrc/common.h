// Device-side helpers shared by the gfx950 kernels: 16-bit storage types, wavefront (64 lanes)
// cross-lane reductions built on DPP, and the launch-parameter block every kernel receives.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lserve {

constexpr int kWave = 64;       // CDNA wavefront width
constexpr int kHeadDim = 128;   // D; every kernel is specialised for it
constexpr int kMaxGroup = 8;    // n = H / Hkv
constexpr int kMaxLogical = 8;  // g = N_P / N_L

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf162_t __attribute__((ext_vector_type(2)));

struct F16 {};
struct BF16 {};

template <class T> struct Elem;

// Two 16-bit elements travel in one 32-bit register; element 0 is the low half.
template <> struct Elem<F16> {
    static __device__ __forceinline__ float lo(uint32_t u) { return (float)__builtin_bit_cast(half2_t, u)[0]; }
    static __device__ __forceinline__ float hi(uint32_t u) { return (float)__builtin_bit_cast(half2_t, u)[1]; }
    // c + a.lo * b.lo + a.hi * b.hi with fp32 accumulation (v_dot2_f32_f16)
    static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), c, false);
    }
    static __device__ __forceinline__ uint32_t pack(float a, float b) {
        half2_t h = {(_Float16)a, (_Float16)b};  // round to nearest even
        return __builtin_bit_cast(uint32_t, h);
    }
};

template <> struct Elem<BF16> {
    static __device__ __forceinline__ float lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
    static __device__ __forceinline__ float hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }
    static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf162_t, a), __builtin_bit_cast(bf162_t, b), c, false);
    }
    static __device__ __forceinline__ uint32_t pack(float a, float b) {
        bf162_t h = {(__bf16)a, (__bf16)b};  // round to nearest even
        return __builtin_bit_cast(uint32_t, h);
    }
};

// ---- DPP cross-lane primitives (row = 16 consecutive lanes) ------------------------------------

template <int Ctrl> __device__ __forceinline__ float dpp_f(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), Ctrl, 0xf, 0xf, true));
}

constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i inside each 8 lanes
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i inside each row

// Sum over the 16 lanes of a row; every lane of the row receives the total.
__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_f<kDppXor1>(x);
    x += dpp_f<kDppXor2>(x);
    x += dpp_f<kDppHalfMirror>(x);
    x += dpp_f<kDppMirror>(x);
    return x;
}

// Reductions across the four rows of a wave (lanes l, l^16, l^32, l^48 hold peers).  gfx950 swaps rows between
// two registers in the vector ALU: v_permlane16_swap exchanges the odd rows of its first operand with the even
// rows of its second, v_permlane32_swap the upper half of the first with the lower half of the second.  With the
// same value in both operands the two results hold, in every lane, the two peers of the pair, so each step is one
// swap and one combine with no trip through the LDS crossbar.  (The elements of the builtin's result are copied
// out before any bit cast: a bit cast applied to the subscripted vector reads element 0 both times.)
typedef unsigned swap_pair_t __attribute__((ext_vector_type(2)));

template <class Op> __device__ __forceinline__ float rows4_combine(float x, Op op) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const swap_pair_t a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned a0 = a[0], a1 = a[1];
    const float y = op(__builtin_bit_cast(float, a0), __builtin_bit_cast(float, a1));  // rows (0,1) and (2,3)
    const unsigned v = __builtin_bit_cast(unsigned, y);
    const swap_pair_t b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    const unsigned b0 = b[0], b1 = b[1];
    return op(__builtin_bit_cast(float, b0), __builtin_bit_cast(float, b1));
}
// Sums of four values over the four rows at once, for the price of one and a half: the odd rows of one value trade
// places with the even rows of another before the two are added, then the halves likewise, and on return row r of the
// result holds the four-row sum of x_r (added as (row 0 + row 1) + (row 2 + row 3), like rows4_sum).
__device__ __forceinline__ float rows4_sum_scatter(float x0, float x1, float x2, float x3) {
    auto swap_add = [](float a, float b, bool halves) {
        const unsigned ua = __builtin_bit_cast(unsigned, a), ub = __builtin_bit_cast(unsigned, b);
        const swap_pair_t p = halves ? __builtin_amdgcn_permlane32_swap(ua, ub, false, false)
                                     : __builtin_amdgcn_permlane16_swap(ua, ub, false, false);
        const unsigned p0 = p[0], p1 = p[1];
        return __builtin_bit_cast(float, p0) + __builtin_bit_cast(float, p1);
    };
    const float t01 = swap_add(x0, x1, false);  // rows 0, 2: pair sums of x0; rows 1, 3: of x1
    const float t23 = swap_add(x2, x3, false);
    return swap_add(t01, t23, true);
}

__device__ __forceinline__ float rows4_sum(float x) {
    return rows4_combine(x, [](float a, float b) { return a + b; });
}
__device__ __forceinline__ float rows4_max(float x) {
    return rows4_combine(x, [](float a, float b) { return fmaxf(a, b); });
}
__device__ __forceinline__ float rows4_min(float x) {
    return rows4_combine(x, [](float a, float b) { return fminf(a, b); });
}

__device__ __forceinline__ float wave_max(float x) {
    x = fmaxf(x, dpp_f<kDppXor1>(x));
    x = fmaxf(x, dpp_f<kDppXor2>(x));
    x = fmaxf(x, dpp_f<kDppHalfMirror>(x));
    x = fmaxf(x, dpp_f<kDppMirror>(x));
    return rows4_max(x);
}

__host__ __device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- parameters ----------------------------------------------------------------------------------

struct LayerParams {
    int H, Hkv, group;       // query heads, KV heads, n = H / Hkv
    int NP, NL, g;           // physical / logical page size, logical pages per physical page
    int sink_pages;          // s = ceil(sink_tokens / NP)
    int local_pages;         // w = ceil(local_tokens / NP)
    unsigned long long streaming_mask;  // bit hk set = KV head hk is a streaming head
    float sm_scale_log2;     // softmax scale * log2(e)
};

struct PagedParams {
    const void *k_pool, *v_pool;      // main pool, pool_heads KV heads per page
    void* stats;
    const int* page_table;
    const int* seq_lens;
    int batch, max_pages, num_pages;
    int pool_heads;
    const void *k_stream, *v_stream;  // bounded pool of the streaming heads (Sec. 3.2), or null
    const int* ring_table;            // [batch][ring]
    int stream_heads, ring;           // heads per page of that pool; ring = s + w slots per sequence
    int kv_bits;                      // 16: K/V rows in 16-bit storage; 8 or 4: quantised pages
};

// Size of one (page, KV head) slab of a K or V pool, in 16-byte units.  16-bit storage: N_P rows of 256
// bytes.  Quantised (Sec. 3.2): N_P rows of 128 codes of `bits` bits, then N_P (scale, zero) pairs of fp16.
__host__ __device__ __forceinline__ constexpr size_t slab_chunks(int NP, int bits) {
    return bits == 16 ? (size_t)NP * (kHeadDim / 8) : (size_t)NP * (kHeadDim * bits / 128) + NP / 4;
}

// Ring slot of the page at position p of a streaming head's sequence: sink pages keep their place,
// local pages reuse w slots in turn.
__device__ __forceinline__ int ring_slot(const LayerParams& lp, int p) {
    return p < lp.sink_pages ? p : lp.sink_pages + (p - lp.sink_pages) % lp.local_pages;
}
// Does KV head hk live in the bounded streaming pool?
__device__ __forceinline__ bool in_stream_pool(const LayerParams& lp, const PagedParams& kv, int hk) {
    return kv.k_stream != nullptr && ((lp.streaming_mask >> hk) & 1ull);
}
// Index of KV head hk inside the pages of the pool that stores it: pools keep their heads in KV-head
// order, so the index is the number of lower heads of the same pool.
__device__ __forceinline__ int pool_rank(const LayerParams& lp, const PagedParams& kv, int hk, bool ring) {
    const unsigned long long below = (1ull << hk) - 1ull;
    if (ring) return __popcll(lp.streaming_mask & below);
    return kv.pool_heads == lp.Hkv ? hk : __popcll(~lp.streaming_mask & below);
}

}  // namespace lserve
