// Block-sparse causal prefill attention (Sec. 3.1, Sec. 3.4) on the gfx950 matrix cores.
//
// Mask tiles are 64 x 64 (query tile x key tile = page).  Dense heads visit every key tile up to
// the diagonal; streaming heads visit only the sink tiles and the local band, so whole tiles
// outside the mask are never loaded.  Only the diagonal tile needs element-wise causal masking.
//
// Mapping to CDNA4: a workgroup of eight wavefronts owns 256 consecutive query rows of one head;
// wavefronts 2t and 2t + 1 own the two 32-row halves of mask tile 4 * block + t.  Two wavefronts
// share each SIMD, so the matrix pipe of one overlaps the softmax arithmetic of the other.  K and
// V tiles are brought into LDS once per workgroup by direct-to-LDS loads, double buffered, and
// consumed by all eight wavefronts.  Scores are computed transposed,
//   S^T (keys x queries) = K (keys x d) * Q^T (d x queries)          v_mfma_f32_32x32x16
// so that a lane owns one query column: the softmax reductions over keys stay inside the lane
// (plus one exchange between the two lane halves), and the exponentiated tile is already in the
// register layout of the B operand of the second product
//   O^T (d x queries) += V^T (d x keys) * P^T (keys x queries).
// V stays as it is in memory, one row per key: the V^T operand is read from the row-major tile with the
// transposing LDS read of gfx950 (ds_read_b64_tr_b16), which hands a lane four keys of one channel, so
// there is no transposition pass and no transposed copy of V.
#include <algorithm>

#include "kernels.h"

namespace lserve {

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf168_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 64;                          // mask tile = key tile = page
constexpr int kPrefillWaves = 8;                   // two per SIMD, each owning 32 query rows
constexpr int kPrefillThreads = kPrefillWaves * kWave;
constexpr int kTilesPerBlock = kPrefillWaves / 2;  // mask tiles of queries per workgroup
constexpr int kRowsPerBlock = kTilesPerBlock * kTile;
constexpr int kDmaLoads = 16 / kPrefillWaves;      // 1 KiB loads per wave, tile and operand
constexpr int kAhead = 4;                          // operand reads in flight ahead of the score products
constexpr int kKRowBytes = 256;                    // K tile row: 128 x 16 bit = 16 chunks of 16 B
constexpr int kVRowBytes = 256;                    // V tile row (one key): the same
constexpr int kKTileBytes = kTile * kKRowBytes;
constexpr int kVTileBytes = kTile * kVRowBytes;

// Tiles reach LDS through direct-to-LDS loads, which place the 64 lanes of an instruction at 64
// consecutive 16-byte slots, so rows cannot be padded.  Bank conflicts are avoided by permuting the
// chunks inside a row instead.  Chunk c of K row r sits at position c ^ (r % 16): sixteen consecutive rows
// then hit sixteen different 16-byte bank groups for any fixed c, which is what the K operand reads (one
// row per lane) need.  Chunk c of V row r sits at position c ^ 4 (r % 4): a transposing read takes, from
// each of four consecutive rows, the same 64 bytes (32 channels), and the four stretches then fall into
// the four 64-byte quarters of the 256 bytes the banks serve per cycle.
__device__ __forceinline__ int k_chunk_pos(int row, int c) { return c ^ (row % 16); }
__device__ __forceinline__ int v_chunk_pos(int row, int c) { return c ^ (4 * (row % 4)); }

// The load itself is written in assembly: left to the compiler it is treated as an access that may
// touch both memory and LDS, and while one is in flight every LDS operand read in the loop waits with
// lgkmcnt(0), exposing the LDS latency in front of the products.  The source address is a wave-uniform
// 64-bit base (scalar registers) plus a 32-bit lane offset; `lds_base` is the wave-uniform LDS byte
// address of the 1 KiB destination and lane l lands at lds_base + 16 l.  Completion is tracked by
// vmcnt only, which dma_wait() drains before the workgroup barrier.
__device__ __forceinline__ void dma_load16(unsigned long long src_base, unsigned lane_offset, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_offset), "s"(src_base), "s"(lds_base) : "memory");
}
// Tells the compiler that a value every lane agrees on can live in scalar registers.
__device__ __forceinline__ unsigned long long uniform64(unsigned long long x) {
    return ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)(x >> 32)) << 32) |
           (unsigned)__builtin_amdgcn_readfirstlane((unsigned)x);
}
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ unsigned lds_address(const void* p) {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void*)p;
}

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

// Chunked prefill over a paged cache (Sec. 2.1, Sec. 3.2).  The cache holds seq_lens[b] tokens of sequence b, in
// any of the forms of PagedParams with 16-bit rows (one pool; dense heads in the main pool and streaming heads in
// their ring of sink + local pages).  With k_new / v_new the queries are n_b new tokens whose K / V arrive
// alongside and have not been written back yet: the cache is their history.  Without, the cache already holds
// the chunk and the queries are its last n_b tokens.
struct PrefillPaged {
    PagedParams kv;
    const uint16_t *k_new, *v_new;  // [total_new][Hkv][D] or null
};

template <class T>
__device__ __forceinline__ uint4 pack8(const float* p) {
    return make_uint4(Elem<T>::pack(p[0], p[1]), Elem<T>::pack(p[2], p[3]), Elem<T>::pack(p[4], p[5]),
                      Elem<T>::pack(p[6], p[7]));
}

// Combine a value with the one held by the same lane of the other 32-lane half of the wave.
// (one swap of the upper half of a register with the lower half of its copy, in the vector ALU)
template <class Op> __device__ __forceinline__ float halves_combine(float x, Op op) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const swap_pair_t p = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned p0 = p[0], p1 = p[1];
    return op(__builtin_bit_cast(float, p0), __builtin_bit_cast(float, p1));
}
__device__ __forceinline__ float halves_max(float x) {
    return halves_combine(x, [](float a, float b) { return fmaxf(a, b); });
}
__device__ __forceinline__ float halves_sum(float x) {
    return halves_combine(x, [](float a, float b) { return a + b; });
}

typedef short short4_t __attribute__((ext_vector_type(4)));
// Transposing LDS read (ds_read_b64_tr_b16).  The sixteen lanes of a row each name four consecutive 16-bit
// elements; lane i receives element i % 4 of the lanes i / 4, i / 4 + 4, i / 4 + 8 and i / 4 + 12.  With lane s
// pointing at channels 4 (s % 4) .. + 3 of key s / 4, lane i ends up with channel i of four consecutive keys.
__device__ __forceinline__ uint2 lds_read_transposed(const unsigned char* p) {
    const short4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) short4_t*)(const __attribute__((address_space(3))) void*)p);
    return __builtin_bit_cast(uint2, v);
}

// Work order of the launch.  Workgroup ids go round-robin over the eight XCDs, each with its own L2.
// Dense heads come first (heaviest query blocks first), streaming heads after.  When the number of
// heads of a class divides 8, an XCD serves a single KV head of that class at a time, so the
// workgroups resident on it (the query heads of one group, neighbouring query blocks) walk the
// same K / V tiles together and share them in that L2.
constexpr int kXcds = 8;
struct HeadClass {
    int heads;          // KV heads of this class
    int slices;         // query-block slices per head spread over XCDs (1 when not swizzled)
    int swizzled;       // 8 % heads == 0
    int items_per_xcd;  // workgroups of this class per XCD
    unsigned char kv_head[64];
};
struct PrefillSchedule {
    HeadClass cls[2];  // dense, streaming
    int qblocks_total; // batch * blocks_per_seq
};

// Decodes workgroup `li` of XCD `xcd` inside a class.  Returns false for padding workgroups.
__device__ __forceinline__ bool decode_work(const HeadClass& hc, int n, int qblocks_total, int xcd, int li, int& hk,
                                            int& hh, int& rank) {
    int hidx;
    if (hc.swizzled) {
        hidx = xcd % hc.heads;
        const int slice = xcd / hc.heads;
        hh = li % n;
        rank = (li / n) * hc.slices + slice;
    } else {
        const int t = li * kXcds + xcd;
        hh = t % n;
        hidx = (t / n) % hc.heads;
        rank = t / (n * hc.heads);
    }
    hk = hc.kv_head[hidx];
    return rank < qblocks_total;
}

// General block mask (Sec. 3.1, Sec. 3.4): per mask and query tile, the ascending list of kept key
// tiles.  A workgroup owns four query tiles; a pre-pass merges their rows into one ascending list of
// (key tile, which of the four query tiles keep it) so that the main loop walks a single list.
struct PrefillMask {
    const int* head_mask;     // [H]: mask of query head h, -1 = analytic mask of the layer description
    const int* q_tile_start;  // [batch + 1]: first row of sequence b inside one mask
    const int* row_ptr;       // [num_masks * rows_per_mask + 1]
    const int* cols;          // key tiles, ascending inside a row
    int rows_per_mask;
    int* blk_list;            // merged lists; the list of a workgroup starts at row_ptr[its first row]
    int* blk_count;           // [num_masks][batch][blocks_per_seq]
};
constexpr int kKeepShift = 24;  // list entry = key tile | keep bits << 24

__global__ __launch_bounds__(kWave) void merge_mask_rows_kernel(PrefillMask mk, const int* __restrict__ cu_seqlens,
                                                                int batch, int blocks_per_seq) {
    extern __shared__ unsigned char keep_bits[];  // one byte per key tile of the sequence
    const int qblk = blockIdx.x, b = blockIdx.y, m = blockIdx.z, lane = threadIdx.x;
    const int len = cu_seqlens[b + 1] - cu_seqlens[b];
    const int n_tiles = ceil_div(len, kTile);
    int* count = mk.blk_count + ((size_t)m * batch + b) * blocks_per_seq + qblk;
    const int iq0 = qblk * kTilesPerBlock;
    if (iq0 >= n_tiles) {
        if (lane == 0) *count = 0;
        return;
    }
    const int rows = min(kTilesPerBlock, n_tiles - iq0);
    const int r0 = m * mk.rows_per_mask + mk.q_tile_start[b] + iq0;
    const int last = min(iq0 + rows, n_tiles);  // key tiles the block can keep: [0, last)
    for (int j = lane; j < last; j += kWave) keep_bits[j] = 0;
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();
    for (int t = 0; t < rows; ++t) {  // one row at a time: no two lanes touch the same byte
        const int lo = mk.row_ptr[r0 + t], hi = mk.row_ptr[r0 + t + 1];
        for (int e = lo + lane; e < hi; e += kWave) {
            const int j = mk.cols[e];
            if (j >= 0 && j <= iq0 + t) keep_bits[j] |= (unsigned char)(1u << t);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_wave_barrier();
    }
    int* dst = mk.blk_list + mk.row_ptr[r0];
    int total = 0;
    for (int j0 = 0; j0 < last; j0 += kWave) {
        const int j = j0 + lane;
        const unsigned bits = j < last ? keep_bits[j] : 0u;
        const unsigned long long live = __ballot(bits != 0);
        if (bits) dst[total + __popcll(live & ((1ull << lane) - 1ull))] = j | (int)(bits << kKeepShift);
        total += __popcll(live);
    }
    if (lane == 0) *count = total;
}

template <class T> struct Ones;
template <> struct Ones<F16> { static constexpr uint32_t pair = 0x3c003c00u; };
template <> struct Ones<BF16> { static constexpr uint32_t pair = 0x3f803f80u; };

enum PrefillMode { kPlain = 0, kMasked = 1, kPaged = 2 };

// BITS: width of the rows in the pages (16, or 8 / 4 for quantised pages, kPaged only).  Quantised tiles cannot take
// the direct-to-LDS path: their codes travel through registers, are turned into the layer's 16-bit type as
// code * scale + zero (fp32, then rounded) and are stored to the same LDS places the direct loads would fill.
template <class T, int MODE, int BITS = 16>
__global__ __launch_bounds__(kPrefillThreads, 512 / kPrefillThreads) void sparse_prefill_kernel(
    LayerParams lp, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int* __restrict__ cu_seqlens, int batch, int blocks_per_seq, uint16_t* __restrict__ out,
    float* __restrict__ lse_out, int total_tokens, PrefillSchedule sched, PrefillMask mk, PrefillPaged pg) {
    constexpr bool MASKED = MODE == kMasked, PAGED = MODE == kPaged, QUANT = BITS != 16;
    static_assert(!QUANT || PAGED, "quantised rows live in pages");
    // Two stages of (K tile, V tile).  Four separate arrays, and a loop unrolled over the two stages,
    // so that the compiler can tell the tile being read from the tile being filled and does not wait
    // for the loads in flight before every operand read.
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds0[kKTileBytes];
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds1[kKTileBytes];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds0[kVTileBytes];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds1[kVTileBytes];

    // heaviest query blocks first; see PrefillSchedule for the XCD-aware order
    const int xcd = blockIdx.x % kXcds;
    int li = blockIdx.x / kXcds, hk, hh, rank;
    bool real;
    if (li < sched.cls[0].items_per_xcd) {
        real = decode_work(sched.cls[0], lp.group, sched.qblocks_total, xcd, li, hk, hh, rank);
    } else {
        li -= sched.cls[0].items_per_xcd;
        real = decode_work(sched.cls[1], lp.group, sched.qblocks_total, xcd, li, hk, hh, rank);
    }
    if (!real) return;
    const int h = hk * lp.group + hh;
    const int b = rank % batch;
    // start: row of the sequence's first query in q / out; len: keys of the sequence; first: position of
    // that first query (0 unless the keys come from a paged cache that already holds earlier tokens)
    const int start = cu_seqlens[b];
    // cached: keys that come from the pages (all of them, or the history of a chunk whose K / V arrive alongside)
    const int cached = PAGED ? pg.kv.seq_lens[b] : 0;
    const int len = PAGED ? (pg.k_new ? cached + (cu_seqlens[b + 1] - start) : cached) : cu_seqlens[b + 1] - start;
    const int first = PAGED ? len - (cu_seqlens[b + 1] - start) : 0;
    const int qblk = first / kRowsPerBlock + blocks_per_seq - 1 - rank / batch;
    if (qblk * kRowsPerBlock >= len) return;
    if (PAGED && first >= len) return;  // a sequence without queries in this chunk

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int n = lane % 32, half = lane / 32;
    const bool streaming = (lp.streaming_mask >> hk) & 1ull;
    const int iq = qblk * kTilesPerBlock + wave / 2;  // this wave's mask tile; the wave owns one half of its rows
    const int row0 = (wave % 2) * 32;    // first row of the wave inside the mask tile
    const int n_qtiles = ceil_div(len, kTile);
    const int iq_last = min(qblk * kTilesPerBlock + kTilesPerBlock - 1, n_qtiles - 1);  // last mask tile of the block that holds rows
    const bool wave_has_rows = iq * kTile + row0 < len && iq * kTile + row0 + 32 > first;

    // key tiles the block visits: [0, sink_end) and [band_begin, iq_last]
    int sink_end, band_begin;
    if (streaming) {
        band_begin = max(0, qblk * kTilesPerBlock - lp.local_pages + 1);
        sink_end = min(lp.sink_pages, band_begin);
    } else {
        band_begin = 0;
        sink_end = 0;
    }
    int n_visit = sink_end + (iq_last - band_begin + 1);
    // a listed mask replaces the closed form: the merged list of this workgroup's four query tiles
    const int* lst = nullptr;
    if (MASKED) {
        const int m = mk.head_mask[h];
        if (m >= 0) {
            lst = mk.blk_list + mk.row_ptr[m * mk.rows_per_mask + mk.q_tile_start[b] + qblk * kTilesPerBlock];
            n_visit = mk.blk_count[((size_t)m * batch + b) * blocks_per_seq + qblk];
        }
    }

    // ---- Q^T operand: lane (n, half) holds Q[row][16 kk + 8 half .. + 8]
    uint4 qreg[8];
    {
        const int row = min(max(iq * kTile + row0 + n, first), len - 1) - first;
        const uint4* src = reinterpret_cast<const uint4*>(q + ((size_t)(start + row) * lp.H + h) * kHeadDim);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qreg[kk] = src[kk * 2 + half];
        // Pin the loads here.  Left alone the compiler sinks them to the loop entry, and because the
        // memory counter completes in order every tile's first product would then wait for that
        // tile's K / V prefetch.
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            asm volatile("" : "+v"(qreg[kk].x), "+v"(qreg[kk].y), "+v"(qreg[kk].z), "+v"(qreg[kk].w));
        // The softmax scale (times log2 e) goes into Q once, so the scores leave the matrix pipe ready for
        // exp2.  The extra rounding of Q to 16 bit moves a logit by about 2^-9 (bf16) or 2^-11 (fp16) of its
        // size times 0.13, an order below the rounding of the softmax weights themselves.
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            uint32_t* w = reinterpret_cast<uint32_t*>(&qreg[kk]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = Elem<T>::pack(Elem<T>::lo(w[i]) * lp.sm_scale_log2, Elem<T>::hi(w[i]) * lp.sm_scale_log2);
        }
    }

    float16_t acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;  // running maximum (scaled, base 2) and sum of this lane's query row
    // The score products start from -m_run instead of 0 (the accumulator input of the first product), so a
    // tile whose maxima do not exceed the running ones needs no subtraction before exp2; 0 while m_run = -inf.
    float16_t neg_m;
#pragma unroll
    for (int i = 0; i < 16; ++i) neg_m[i] = 0.f;

    // ---- staging: every wave issues two direct-to-LDS loads of 1 KiB per tile and operand
    // contiguous keys: tile jt starts jt * 64 rows after the sequence's first row; paged keys: tile jt is the
    // slab of (its page, hk) in the pool the head lives in, rows 256 bytes apart; keys of a chunk that has not
    // been written back: row u - cached of the chunk's own K / V
    const bool ring = PAGED && in_stream_pool(lp, pg.kv, hk);  // a streaming head kept in its bounded pool
    const int heads_in_pool = PAGED ? (ring ? pg.kv.stream_heads : pg.kv.pool_heads) : lp.Hkv;
    constexpr size_t kSlabBytes = slab_chunks(kTile, BITS) * 16;  // one (page, head) of a pool
    const size_t slab_in_page = PAGED ? (size_t)pool_rank(lp, pg.kv, hk, ring) * (kSlabBytes / 2) : 0;  // in 16-bit units
    const uint16_t* kbase = PAGED ? reinterpret_cast<const uint16_t*>(ring ? pg.kv.k_stream : pg.kv.k_pool) + slab_in_page
                                  : k + ((size_t)start * lp.Hkv + hk) * kHeadDim;
    const uint16_t* vbase = PAGED ? reinterpret_cast<const uint16_t*>(ring ? pg.kv.v_stream : pg.kv.v_pool) + slab_in_page
                                  : v + ((size_t)start * lp.Hkv + hk) * kHeadDim;
    const int* page_row = !PAGED ? nullptr
                          : ring ? pg.kv.ring_table + (size_t)b * pg.kv.ring
                                 : pg.kv.page_table + (size_t)b * pg.kv.max_pages;
    // page of key tile jt, for tiles that hold cached keys (0 otherwise: never used)
    auto page_of = [&](int jt) {
        if (!PAGED || jt * kTile >= cached) return 0;
        return page_row[ring ? ring_slot(lp, jt) : jt];
    };
    // lane `lane` of load i of this wave fills slot (2 wave + i) * 64 + lane of the tile, i.e. position lane % 16
    // of row 4 (2 wave + i) + lane / 16.  Addresses are a wave-uniform 64-bit tile base (scalar arithmetic) plus a
    // 32-bit lane offset that does not depend on the tile, except in the last tile of a sequence, where rows
    // past the end read the last row again (finite values; their softmax weights are 0).
    const unsigned seq_row_bytes = (unsigned)__builtin_amdgcn_readfirstlane(lp.Hkv * kHeadDim * 2);  // [token][Hkv][D]
    const unsigned k_row_bytes = PAGED ? kHeadDim * 2u : seq_row_bytes;
    const unsigned long long k_page_bytes = (unsigned long long)heads_in_pool * kSlabBytes;
    const int krow0 = wave * (4 * kDmaLoads) + lane / 16;  // K row of load 0; load i takes row + 4 i
    unsigned kofs[kDmaLoads], vofs[kDmaLoads];
#pragma unroll
    for (int i = 0; i < kDmaLoads; ++i) {
        kofs[i] = (unsigned)(krow0 + 4 * i) * k_row_bytes + k_chunk_pos(krow0 + 4 * i, lane % 16) * 16;  // an involution
        vofs[i] = (unsigned)(krow0 + 4 * i) * k_row_bytes + v_chunk_pos(krow0 + 4 * i, lane % 16) * 16;  // likewise
    }
    const unsigned lds_wave = (unsigned)__builtin_amdgcn_readfirstlane(wave * kDmaLoads * 1024);
    const unsigned long long kbase_u = uniform64((unsigned long long)kbase), vbase_u = uniform64((unsigned long long)vbase);
    // the chunk's own rows, addressed from its first token (the row of position `cached`)
    const unsigned long long knew_u =
        uniform64((unsigned long long)(PAGED && pg.k_new ? pg.k_new + ((size_t)start * lp.Hkv + hk) * kHeadDim : nullptr));
    const unsigned long long vnew_u =
        uniform64((unsigned long long)(PAGED && pg.v_new ? pg.v_new + ((size_t)start * lp.Hkv + hk) * kHeadDim : nullptr));
    const int len_u = __builtin_amdgcn_readfirstlane(len), cached_u = __builtin_amdgcn_readfirstlane(cached);
    // quantised rows on their way through registers: per load the codes of this lane's 16-byte place (8 channels) of
    // K and of V, the (scale, zero) pairs of the row, and whether the lane's row comes from the pages at all
    constexpr int kRowCodeBytes = kHeadDim * BITS / 8, kPlaceCodeBytes = BITS;  // per row; per 8 channels
    uint2 staged_k[kDmaLoads], staged_v[kDmaLoads];
    uint32_t staged_ksz[kDmaLoads], staged_vsz[kDmaLoads];
    int staged_from = 0, staged_left = 1;  // of the tile in flight: rows that come from the pages; rows it has
    auto fetch = [&](unsigned char* kd, unsigned char* vd, int jt, int phys) {
        jt = __builtin_amdgcn_readfirstlane(jt);
        if constexpr (QUANT) {
            const int rows_left = len_u - jt * kTile;
            const int from_pages = cached_u - jt * kTile;  // rows of the tile below this come from the pages
            staged_from = from_pages;
            staged_left = rows_left;
            const unsigned char* kslab = reinterpret_cast<const unsigned char*>(kbase) +
                                         (size_t)(unsigned)__builtin_amdgcn_readfirstlane(phys) * k_page_bytes;
            const unsigned char* vslab = kslab - reinterpret_cast<const unsigned char*>(kbase) +
                                         reinterpret_cast<const unsigned char*>(vbase);
            const unsigned long long shift = (unsigned long long)((long long)jt * kTile - cached_u) * seq_row_bytes;
#pragma unroll
            for (int i = 0; i < kDmaLoads; ++i) {
                const int row = krow0 + 4 * i, r = min(row, rows_left - 1);
                const int kplace = k_chunk_pos(row, lane % 16), vplace = v_chunk_pos(row, lane % 16);
                if (r < from_pages) {
                    const unsigned char* kr = kslab + (size_t)r * kRowCodeBytes + kplace * kPlaceCodeBytes;
                    const unsigned char* vr = vslab + (size_t)r * kRowCodeBytes + vplace * kPlaceCodeBytes;
                    if constexpr (BITS == 8) {
                        staged_k[i] = *reinterpret_cast<const uint2*>(kr);
                        staged_v[i] = *reinterpret_cast<const uint2*>(vr);
                    } else {
                        staged_k[i] = make_uint2(*reinterpret_cast<const uint32_t*>(kr), 0u);
                        staged_v[i] = make_uint2(*reinterpret_cast<const uint32_t*>(vr), 0u);
                    }
                    staged_ksz[i] = reinterpret_cast<const uint32_t*>(kslab + kTile * kRowCodeBytes)[r];
                    staged_vsz[i] = reinterpret_cast<const uint32_t*>(vslab + kTile * kRowCodeBytes)[r];
                } else {  // a row of the chunk: 16-bit, straight to LDS
                    dma_load16(knew_u + shift, (unsigned)r * seq_row_bytes + kplace * 16,
                               __builtin_amdgcn_readfirstlane(lds_address(kd) + lds_wave + i * 1024));
                    dma_load16(vnew_u + shift, (unsigned)r * seq_row_bytes + vplace * 16,
                               __builtin_amdgcn_readfirstlane(lds_address(vd) + lds_wave + i * 1024));
                }
            }
            return;
        }
        const unsigned long long ktile =
            PAGED ? kbase_u + (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane(phys) * k_page_bytes
                  : kbase_u + (unsigned long long)jt * (kTile * k_row_bytes);
        const unsigned long long vtile = ktile - kbase_u + vbase_u;  // K and V are laid out alike
        // Rows at or past the sequence length must not be read as they are: a page may hold anything there, and
        // although their weights are 0 a non-finite value would still poison the second product.
        const int rows_left = len_u - jt * kTile;
        // rows of the tile below `from_pages` come from the page, the others from the chunk's own K / V
        const int from_pages = PAGED ? cached_u - jt * kTile : kTile;
        if (!PAGED || from_pages >= min(rows_left, kTile)) {
#pragma unroll
            for (int i = 0; i < kDmaLoads; ++i) {
                unsigned ko = kofs[i], vo = vofs[i];
                if (rows_left < kTile) {
                    const int row = krow0 + 4 * i;
                    ko = (unsigned)min(row, rows_left - 1) * k_row_bytes + k_chunk_pos(row, lane % 16) * 16;
                    vo = (unsigned)min(row, rows_left - 1) * k_row_bytes + v_chunk_pos(row, lane % 16) * 16;
                }
                dma_load16(ktile, ko, __builtin_amdgcn_readfirstlane(lds_address(kd) + lds_wave + i * 1024));
                dma_load16(vtile, vo, __builtin_amdgcn_readfirstlane(lds_address(vd) + lds_wave + i * 1024));
            }
        } else {
            // the tile holds rows of the chunk: row r of the tile is the chunk's token jt * 64 + r - cached
            const unsigned long long shift = (unsigned long long)((long long)jt * kTile - cached_u) * seq_row_bytes;
            const unsigned long long ktile_new = knew_u + shift, vtile_new = vnew_u + shift;
#pragma unroll
            for (int i = 0; i < kDmaLoads; ++i) {
                const int row = krow0 + 4 * i, r = min(row, rows_left - 1);
                const unsigned kc = k_chunk_pos(row, lane % 16) * 16, vc = v_chunk_pos(row, lane % 16) * 16;
                const unsigned lds_k = __builtin_amdgcn_readfirstlane(lds_address(kd) + lds_wave + i * 1024);
                const unsigned lds_v = __builtin_amdgcn_readfirstlane(lds_address(vd) + lds_wave + i * 1024);
                if (r < from_pages) {  // only in the one tile that straddles the end of the cache
                    dma_load16(ktile, (unsigned)r * k_row_bytes + kc, lds_k);
                    dma_load16(vtile, (unsigned)r * k_row_bytes + vc, lds_v);
                } else {
                    dma_load16(ktile_new, (unsigned)r * seq_row_bytes + kc, lds_k);
                    dma_load16(vtile_new, (unsigned)r * seq_row_bytes + vc, lds_v);
                }
            }
        }
    };
    // Entry `it` of the walk: key tile in the low bits; with a listed mask also which query tiles keep it.
    auto entry_of = [&](int it) {
        if (MASKED && lst) return lst[it];
        return it < sink_end ? it : band_begin + (it - sink_end);
    };
    int e_cur = n_visit > 0 ? entry_of(0) : 0, e_nxt = n_visit > 1 ? entry_of(1) : 0;
    // physical pages of the tiles to come, looked up two steps ahead of the loads that need them
    int ph_cur = n_visit > 0 ? page_of(e_cur) : 0, ph_nxt = n_visit > 1 ? page_of(e_nxt) : 0;

    // loop-invariant operand offsets of this lane inside a tile
    int koff[8], voff[4];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) koff[kk] = n * kKRowBytes + k_chunk_pos(n, kk * 2 + half) * 16;
    // V^T operand of (channel block db, 16-key step, half u of the lane's 8 keys): the lane's row of sixteen names
    // keys 16 step + 8 u + 4 half + s / 4 (s = lane % 16) and channels 32 db + 16 (n / 16) + 4 (s % 4) .. + 3, which
    // after the exchange leaves lane (n, half) with channel 32 db + n of keys 16 step + 8 u + 4 half + 0 .. 3: the
    // keys its weights P^T[8 half + 4 u .. + 3] belong to.  Per db the lane part of the address is fixed; step and u
    // add (4 step + 2 u) KiB.
#pragma unroll
    for (int db = 0; db < 4; ++db) {
        const int s16 = lane % 16, rr = s16 / 4;
        const int chunk = 4 * db + 2 * (n / 16) + (s16 % 4) / 2;
        voff[db] = half * 1024 + rr * kVRowBytes + v_chunk_pos(rr, chunk) * 16 + 8 * (s16 % 2);
    }

    // Quantised rows fetched for the tile in flight: eight codes -> code * scale + zero -> eight 16-bit values at the
    // lane's place of the row in LDS (the place a direct load of the same row would have filled).
    auto dequantise8 = [&](uint2 codes, uint32_t scale_zero) {
        const half2_t sz = __builtin_bit_cast(half2_t, scale_zero);
        const float scale = (float)sz[0], zero = (float)sz[1];
        uint32_t lo = codes.x, hi = codes.y;  // channels 0..3 and 4..7, one byte each
        if constexpr (BITS == 4) {
            hi = (codes.x >> 4) & 0x0f0f0f0fu;
            lo = codes.x & 0x0f0f0f0fu;
        }
        float x[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[j] = __builtin_fmaf((float)((lo >> (8 * j)) & 0xffu), scale, zero);
            x[4 + j] = __builtin_fmaf((float)((hi >> (8 * j)) & 0xffu), scale, zero);
        }
        return pack8<T>(x);
    };
    auto store_staged = [&](unsigned char* kd, unsigned char* vd) {
        if constexpr (QUANT) {
            if (staged_from <= 0) return;
#pragma unroll
            for (int i = 0; i < kDmaLoads; ++i) {
                if (min(krow0 + 4 * i, staged_left - 1) < staged_from) {  // the lanes that fetch() gave codes
                    *reinterpret_cast<uint4*>(kd + lds_wave + i * 1024 + lane * 16) = dequantise8(staged_k[i], staged_ksz[i]);
                    *reinterpret_cast<uint4*>(vd + lds_wave + i * 1024 + lane * 16) = dequantise8(staged_v[i], staged_vsz[i]);
                }
            }
        }
    };

    auto tile_step = [&](int it, const unsigned char* ks, const unsigned char* vs, unsigned char* kd, unsigned char* vd) {
        const int e_new = it + 2 < n_visit ? entry_of(it + 2) : 0;  // requested two steps ahead of its use
        const int ph_new = it + 2 < n_visit ? page_of(e_new) : 0;
        const int jt = e_cur & ((1 << kKeepShift) - 1);
        if (it + 1 < n_visit) fetch(kd, vd, e_nxt & ((1 << kKeepShift) - 1), ph_nxt);
        ph_nxt = ph_new;
        // does this wave's mask tile keep key tile jt?
        bool keep = wave_has_rows && jt <= iq;
        if (MASKED && lst)
            keep = keep && ((e_cur >> (kKeepShift + wave / 2)) & 1);
        else if (streaming)
            keep = keep && (jt < lp.sink_pages || jt > iq - lp.local_pages);
        e_cur = e_nxt;
        e_nxt = e_new;
        if (keep) {
            const bool diagonal = jt == iq;
            // S^T for the 64 keys of the tile, two blocks of 32 keys.  All operand reads of a block are
            // issued before its products so that LDS latency is paid once, and the two blocks'
            // accumulation chains alternate in the matrix pipe.
            __builtin_amdgcn_s_setprio(2);  // products first: the other wavefront of the SIMD fills in with softmax work
            float16_t s[2];
            uint4 ka[8][2];
#pragma unroll
            for (int kk = 0; kk < 8; ++kk)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    ka[kk][kb] = *reinterpret_cast<const uint4*>(ks + kb * 32 * kKRowBytes + koff[kk]);
            s[0] = Mfma<T>::run(ka[0][0], qreg[0], neg_m);
            s[1] = Mfma<T>::run(ka[0][1], qreg[0], neg_m);
#pragma unroll
            for (int kk = 1; kk < 8; ++kk) {
                s[0] = Mfma<T>::run(ka[kk][0], qreg[kk], s[0]);
                s[1] = Mfma<T>::run(ka[kk][1], qreg[kk], s[1]);
            }
            // schedule: operand reads run four ahead of the products that consume them
            __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
            for (int u = 0; u < 16 - kAhead; ++u) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
            __builtin_amdgcn_s_setprio(0);
            if (diagonal) {  // causal mask inside the diagonal tile
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kb * 32 + 8 * (i / 4) + 4 * half + (i % 4);
                        if (key > row0 + n) s[kb][i] = -INFINITY;
                    }
            }
            // online softmax of this lane's query row (its keys are split between the two lane halves)
            float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[0][i]), s[1][i]);  // v_max3_f32
            mx = halves_max(mx);  // relative to the running maximum (to 0 before the first kept tile)
            if (__any(mx > 0.f || m_run == -INFINITY)) {  // some row's maximum moved: subtract and rescale
                const float m_base = m_run == -INFINITY ? 0.f : m_run;
                const float m_new = fmaxf(m_run, m_base + mx);
                const float delta = m_new - m_base;                         // 0 for rows whose maximum stayed
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // exp2(-inf) = 0 on the first tile
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[db][i] *= alpha;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[kb][i] -= delta;
                m_run = m_new;
#pragma unroll
                for (int i = 0; i < 16; ++i) neg_m[i] = -m_new;
            }
            uint4 pb[2][2];  // P^T packed to 16 bit: [key block][16-key step]
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                float pf[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) pf[i] = __builtin_amdgcn_exp2f(s[kb][i]);
                pb[kb][0] = pack8<T>(pf);
                pb[kb][1] = pack8<T>(pf + 8);
                // row sum from the rounded weights, the same values the second product uses
                const uint32_t w[8] = {pb[kb][0].x, pb[kb][0].y, pb[kb][0].z, pb[kb][0].w,
                                       pb[kb][1].x, pb[kb][1].y, pb[kb][1].z, pb[kb][1].w};
#pragma unroll
                for (int u = 0; u < 8; ++u) l_run = Elem<T>::dot2(w[u], Ones<T>::pair, l_run);
            }
            // O^T += V^T * P^T, 16 keys per instruction; operand reads run one step ahead
#pragma unroll
            for (int step = 0; step < 4; ++step) {
                const int kb = step / 2, j = step % 2;
                uint4 va[4];
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const uint2 lo = lds_read_transposed(vs + (4 * step) * 1024 + voff[db]);
                    const uint2 hi = lds_read_transposed(vs + (4 * step + 2) * 1024 + voff[db]);
                    va[db] = make_uint4(lo.x, lo.y, hi.x, hi.y);
                }
#pragma unroll
                for (int db = 0; db < 4; ++db) acc[db] = Mfma<T>::run(va[db], pb[kb][j], acc[db]);
            }
        }
        if (it + 1 < n_visit) store_staged(kd, vd);
        dma_wait();
        __syncthreads();  // the next tile has landed and this one is free
    };

    if (n_visit > 0) {
        fetch(k_lds0, v_lds0, e_cur & ((1 << kKeepShift) - 1), ph_cur);
        store_staged(k_lds0, v_lds0);
    }
    dma_wait();
    __syncthreads();
    for (int it = 0; it < n_visit; it += 2) {
        tile_step(it, k_lds0, v_lds0, k_lds1, v_lds1);
        if (it + 1 >= n_visit) break;
        tile_step(it + 1, k_lds1, v_lds1, k_lds0, v_lds0);
    }

    if (!wave_has_rows) return;
    // ---- epilogue: lane (n, half) holds O^T[d][q] for d = 32 db + 8 (i / 4) + 4 half + i % 4
    const float lt = halves_sum(l_run);
    const int pos = iq * kTile + row0 + n;
    if (pos >= len || pos < first) return;
    const int row = pos - first;
    const float inv = lt > 0.f ? 1.f / lt : 0.f;  // a row that keeps nothing (possible with a listed mask) gives 0
    uint16_t* dst = out + ((size_t)(start + row) * lp.H + h) * kHeadDim;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const int d = db * 32 + 8 * g4 + 4 * half;
            uint2 w;
            w.x = Elem<T>::pack(acc[db][4 * g4] * inv, acc[db][4 * g4 + 1] * inv);
            w.y = Elem<T>::pack(acc[db][4 * g4 + 2] * inv, acc[db][4 * g4 + 3] * inv);
            *reinterpret_cast<uint2*>(dst + d) = w;
        }
    if (lse_out && half == 0)
        lse_out[(size_t)h * total_tokens + start + row] = lt > 0.f ? (m_run + __builtin_amdgcn_logf(lt)) * kLn2 : -INFINITY;
}

PrefillSchedule make_schedule(const LayerParams& lp, int blocks_per_seq, int batch) {
    PrefillSchedule sched;
    sched.qblocks_total = blocks_per_seq * batch;
    for (int c = 0; c < 2; ++c) {
        HeadClass& hc = sched.cls[c];
        hc.heads = 0;
        for (int hk = 0; hk < lp.Hkv; ++hk)
            if ((int)((lp.streaming_mask >> hk) & 1ull) == c) hc.kv_head[hc.heads++] = (unsigned char)hk;
        hc.swizzled = hc.heads > 0 && kXcds % hc.heads == 0;
        hc.slices = hc.swizzled ? kXcds / hc.heads : 1;
        if (hc.heads == 0)
            hc.items_per_xcd = 0;
        else if (hc.swizzled)
            hc.items_per_xcd = lp.group * ((sched.qblocks_total + hc.slices - 1) / hc.slices);
        else
            hc.items_per_xcd = (hc.heads * lp.group * sched.qblocks_total + kXcds - 1) / kXcds;
    }
    return sched;
}

size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

template <class T>
hipError_t launch_prefill(const LayerParams& lp, const void* q, const void* k, const void* v, const int* cu_seqlens,
                          int batch, int total_tokens, int max_seqlen, void* out, float* lse_out, void* workspace,
                          const PrefillMaskArgs* mask, hipStream_t stream) {
    const int max_tiles = (max_seqlen + kTile - 1) / kTile;
    hipError_t e = hipSuccess;
    const int blocks_per_seq = (max_seqlen + kRowsPerBlock - 1) / kRowsPerBlock;
    PrefillMask mk = {};
    if (mask) {
        unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
        mk.head_mask = mask->head_mask;
        mk.q_tile_start = mask->q_tile_start;
        mk.row_ptr = mask->row_ptr;
        mk.cols = mask->cols;
        mk.rows_per_mask = mask->rows_per_mask;
        mk.blk_list = reinterpret_cast<int*>(ws);
        mk.blk_count = reinterpret_cast<int*>(ws + align16((size_t)mask->nnz * sizeof(int)));
        hipLaunchKernelGGL(merge_mask_rows_kernel, dim3(blocks_per_seq, batch, mask->num_masks), dim3(kWave),
                           (size_t)align16(max_tiles), stream, mk, cu_seqlens, batch, blocks_per_seq);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const PrefillSchedule sched = make_schedule(lp, blocks_per_seq, batch);
    const int grid = kXcds * (sched.cls[0].items_per_xcd + sched.cls[1].items_per_xcd);
    const PrefillPaged pg = {};  // not read by these instantiations
    if (mask)
        hipLaunchKernelGGL((sparse_prefill_kernel<T, kMasked>), dim3(grid), dim3(kPrefillThreads), 0, stream, lp,
                           reinterpret_cast<const uint16_t*>(q), reinterpret_cast<const uint16_t*>(k),
                           reinterpret_cast<const uint16_t*>(v), cu_seqlens, batch, blocks_per_seq,
                           reinterpret_cast<uint16_t*>(out), lse_out, total_tokens, sched, mk, pg);
    else
        hipLaunchKernelGGL((sparse_prefill_kernel<T, kPlain>), dim3(grid), dim3(kPrefillThreads), 0, stream, lp,
                           reinterpret_cast<const uint16_t*>(q), reinterpret_cast<const uint16_t*>(k),
                           reinterpret_cast<const uint16_t*>(v), cu_seqlens, batch, blocks_per_seq,
                           reinterpret_cast<uint16_t*>(out), lse_out, total_tokens, sched, mk, pg);
    return hipGetLastError();
}

template <class T>
hipError_t launch_prefill_paged(const LayerParams& lp, const PagedParams& kv, const void* q, const void* k_new,
                                const void* v_new, const int* cu_q, int total_new, int max_new_per_seq, int max_seqlen,
                                void* out, float* lse_out, void* workspace, hipStream_t stream) {
    PrefillPaged pg;
    pg.kv = kv;
    pg.k_new = reinterpret_cast<const uint16_t*>(k_new);
    pg.v_new = reinterpret_cast<const uint16_t*>(v_new);
    (void)workspace;
    (void)max_seqlen;
    // the chunk's rows start anywhere inside a 256-row block: one block more than the chunk length needs
    const int blocks_per_seq = (max_new_per_seq + kRowsPerBlock - 1) / kRowsPerBlock + 1;
    const PrefillSchedule sched = make_schedule(lp, blocks_per_seq, kv.batch);
    const int grid = kXcds * (sched.cls[0].items_per_xcd + sched.cls[1].items_per_xcd);
    const PrefillMask mk = {};
#define LSERVE_PREFILL_PAGED(BITS)                                                                                     \
    hipLaunchKernelGGL((sparse_prefill_kernel<T, kPaged, BITS>), dim3(grid), dim3(kPrefillThreads), 0, stream, lp,     \
                       reinterpret_cast<const uint16_t*>(q), nullptr, nullptr, cu_q, kv.batch, blocks_per_seq,         \
                       reinterpret_cast<uint16_t*>(out), lse_out, total_new, sched, mk, pg)
    if (kv.kv_bits == 8)
        LSERVE_PREFILL_PAGED(8);
    else if (kv.kv_bits == 4)
        LSERVE_PREFILL_PAGED(4);
    else
        LSERVE_PREFILL_PAGED(16);
#undef LSERVE_PREFILL_PAGED
    return hipGetLastError();
}

}  // namespace

hipError_t preload_prefill_kernels() {
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&merge_mask_rows_kernel));
}

size_t paged_prefill_workspace_bytes(const LayerParams& lp, int batch, int max_pages) {
    (void)lp;
    (void)batch;
    (void)max_pages;
    return 0;  // keys and values are read from the pages as they are
}

hipError_t launch_sparse_prefill_paged(int dtype, const LayerParams& lp, const PagedParams& kv, const void* q,
                                       const void* k_new, const void* v_new, const int* cu_q, int total_new,
                                       int max_new_per_seq, int max_seqlen, void* out, float* lse_out, void* workspace,
                                       hipStream_t stream) {
    return dtype == 0 ? launch_prefill_paged<F16>(lp, kv, q, k_new, v_new, cu_q, total_new, max_new_per_seq, max_seqlen,
                                                  out, lse_out, workspace, stream)
                      : launch_prefill_paged<BF16>(lp, kv, q, k_new, v_new, cu_q, total_new, max_new_per_seq, max_seqlen,
                                                   out, lse_out, workspace, stream);
}

size_t prefill_workspace_bytes(const LayerParams& lp, int total_tokens, int batch) {
    (void)lp;
    (void)total_tokens;
    (void)batch;
    return 0;  // Q, K and V are read where they are
}

// The merged tile lists (at most one entry per mask entry), then one count per (mask, sequence, workgroup of
// query rows).
size_t masked_prefill_workspace_bytes(const LayerParams& lp, int total_tokens, int batch, int max_seqlen, int num_masks,
                                      int nnz) {
    const int blocks_per_seq = (max_seqlen + kRowsPerBlock - 1) / kRowsPerBlock;
    (void)lp;
    (void)total_tokens;
    return align16((size_t)nnz * sizeof(int)) +
           align16((size_t)num_masks * batch * blocks_per_seq * sizeof(int));
}

hipError_t launch_sparse_prefill(int dtype, const LayerParams& lp, const void* q, const void* k, const void* v,
                                 const int* cu_seqlens, int batch, int total_tokens, int max_seqlen, void* out,
                                 float* lse_out, void* workspace, const PrefillMaskArgs* mask, hipStream_t stream) {
    return dtype == 0 ? launch_prefill<F16>(lp, q, k, v, cu_seqlens, batch, total_tokens, max_seqlen, out, lse_out,
                                            workspace, mask, stream)
                      : launch_prefill<BF16>(lp, q, k, v, cu_seqlens, batch, total_tokens, max_seqlen, out, lse_out,
                                             workspace, mask, stream);
}

}  // namespace lserve
