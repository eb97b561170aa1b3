// np_lookup_bwd: per-key gradient = sum over the key's lookups of the upstream gradient of the bag (or
// sequence position) the lookup belongs to (Section II-A / IV-A: gradients are aggregated per key at the
// owner; Eq. (2) sums the per-sample gradients of a key over the batch).
//
// A deterministic segmented reduction over np_dedup's occurrence lists, balanced under any skew:
//
//   bwd_prepare    two independent preparations in one launch:
//                  the bag map, a bitmap of bag starts plus one bag index per 64 lookups (lookup -> bag in one 16-byte
//                  read), and, for every tile of 256 consecutive sorted positions, the key segment its first position is in
//   bwd_order      execution order of the tiles (it changes no result, only which dY rows are in cache): the lookups
//                  of one key are spread evenly over the bags, so the tiles of all long segments are run sorted by
//                  their relative position inside their segment, one contiguous range of relative positions per
//                  die; tiles running at the same time then read the same band of dY rows from L2 / Infinity
//                  Cache instead of once per lookup from HBM.  One stable partition pass over the tile list.
//   bwd_main       one block per tile.  Every thread prepares one position (dY row, weight, head/tail flags
//                  of its segment); then each LPR-lane group walks its LPR positions in order, several dY row
//                  loads in flight, and closes a running sum whenever a segment ends.  Sums of segments that
//                  lie inside one group's strip go straight to grads.  Sums cut by a strip edge are combined
//                  across the groups of the block in strip order; sums cut by a tile edge are parked in the
//                  workspace as the tile's "left" (continues from an earlier tile) and "right" (continues
//                  into later tiles) partials.
//   bwd_fixup      the tile where a cut segment starts adds its right partial and the left partials of the
//                  following tiles in tile order: one group per tile for short chains, one block per listed
//                  long chain (bwd_main lists them) with a fixed split of the chain over the block.
//
// Two alternatives sit behind np_tune_set, off unless asked for (both measured slower in one call on an MI355X, both give
// the same bits): "bwd_row_index" (bwd_rows resolves the upstream-gradient row of every sorted position ahead of the
// reduction, which then requests its first rows before it knows its tile) and "bwd_singles_by_bag" (keys with one lookup
// are copied bag by bag, bwd_main skips them).
//
// The order of every floating-point addition is a function of occ_offsets alone: no atomics, no dependence
// on scheduling, so two runs give the same bits.  A hot key with millions of lookups costs the same per
// lookup as a cold one.
#include "np_partition.hpp"

namespace np {

constexpr int kBwdTile = 256;
constexpr int kFixupShort = 8;  // chains of up to this many left partials are summed by one group, longer ones by a block
#ifndef NP_BWD_UNROLL
#define NP_BWD_UNROLL 8
#endif
constexpr int kBwdUnroll = NP_BWD_UNROLL;  // dY row loads in flight per lane
constexpr int kOrderBuckets = 1024;   // relative positions inside a long segment
#ifndef NP_ORDER_MIN_COUNT
#define NP_ORDER_MIN_COUNT 2048
#endif
#ifndef NP_ORDER_XCD_SPLIT
#define NP_ORDER_XCD_SPLIT 1
#endif
#ifndef NP_ORDER_INTERLEAVE
#define NP_ORDER_INTERLEAVE 0  // measured on 42 M lookups, dim 64: the two kinds of tiles interleaved 2.03 ms, one after the other 1.97 ms
#endif
constexpr int kOrderMinCount = NP_ORDER_MIN_COUNT;       // segments at least this long take part in the locality order

// One entry per 64 consecutive lookups: where bags start inside the block and which bag the block begins in.
// 16 bytes per 64 lookups (n/4 bytes in all), so the random reads of bwd_main mostly stay in L2 / Infinity Cache.
struct __align__(16) BagMapEntry {
    uint64_t starts;  // bit k (1..63): a bag starts at lookup 64w + k
    int32_t bag0;     // bag holding lookup 64w; sign bit: an empty bag also starts inside the block -> walk bag_offsets
    int32_t start0;   // bag_offsets[bag0]
};

__device__ __forceinline__ void bagmap_entry(int w, const int32_t* __restrict__ bag_offsets, int num_bags, int n,
                                              BagMapEntry* __restrict__ map) {
    const int64_t base64 = static_cast<int64_t>(w) * 64;
    if (base64 >= n) return;
    const int base = static_cast<int>(base64);
    int lo = 0, hi = num_bags;  // last bag in [lo, hi) that starts at or before base; it is non-empty and holds base
    while (hi - lo > 1) {
        const int mid = lo + (hi - lo) / 2;
        if (bag_offsets[mid] <= base) lo = mid;
        else hi = mid;
    }
    const int last = n - 1 - base < 63 ? n - 1 : base + 63;
    uint64_t bits = 0;
    bool twice = false;
    for (int b = lo + 1; b < num_bags; ++b) {
        const int o = bag_offsets[b];
        if (o > last) break;
        const uint64_t m = 1ull << (o - base);
        twice |= (bits & m) != 0;
        bits |= m;
    }
    BagMapEntry e;
    e.starts = bits;
    e.bag0 = twice ? (lo | static_cast<int32_t>(0x80000000u)) : lo;
    e.start0 = bag_offsets[lo];
    map[w] = e;
}

// Bag of lookup j and the first lookup of that bag, from the map entry of j's block of 64 lookups.
__device__ __forceinline__ void bag_from_entry(const BagMapEntry& e, const int32_t* __restrict__ bag_offsets, int j, int& bag, int& start) {
    const int k = j & 63;
    const uint64_t m = e.starts & ((2ull << k) - 1ull);  // starts at or before j (bit 0 is never set)
    bag = (e.bag0 & 0x7FFFFFFF) + __popcll(m);
    start = m ? (j - k + 63 - __clzll(static_cast<long long>(m))) : e.start0;
    if (e.bag0 < 0) {  // an empty bag starts in this block: the bit count misses it, walk the offsets instead
        int b = e.bag0 & 0x7FFFFFFF;
        while (bag_offsets[b + 1] <= j) ++b;
        bag = b;
        start = bag_offsets[b];
    }
}

__device__ __forceinline__ void bag_of_lookup(const BagMapEntry* __restrict__ map, const int32_t* __restrict__ bag_offsets, int j,
                                              int& bag, int& start) {
    bag_from_entry(map[j >> 6], bag_offsets, j, bag, start);
}

__device__ __forceinline__ void tile_first_segment(int t, const int32_t* __restrict__ occ_offsets, const int32_t* __restrict__ d_num_unique,
                                                   int n, int num_tiles, int32_t* __restrict__ tile_seg0) {
    if (t >= num_tiles) return;
    const int pos = t * kBwdTile;
    int lo = 0, hi = device_count(d_num_unique, n);  // U <= n; the answer is the last u in [lo, hi) with occ_offsets[u] <= pos
    while (hi - lo > 1) {
        const int mid = lo + (hi - lo) / 2;
        if (occ_offsets[mid] <= pos) lo = mid;
        else hi = mid;
    }
    tile_seg0[t] = lo;
}

// The two preparations that depend on nothing but the batch's index arrays, in one launch: the first map_blocks blocks
// write the bag map (one entry per thread), the rest find the first segment of every tile (one tile per thread).
__global__ void __launch_bounds__(256)
bwd_prepare_kernel(const int32_t* __restrict__ bag_offsets, int num_bags, int n, BagMapEntry* __restrict__ map, int map_blocks,
                   const int32_t* __restrict__ occ_offsets, const int32_t* __restrict__ d_num_unique, int num_tiles,
                   int32_t* __restrict__ tile_seg0) {
    if (static_cast<int>(blockIdx.x) < map_blocks)
        bagmap_entry(blockIdx.x * 256 + threadIdx.x, bag_offsets, num_bags, n, map);
    else
        tile_first_segment((blockIdx.x - map_blocks) * 256 + threadIdx.x, occ_offsets, d_num_unique, n, num_tiles, tile_seg0);
}

// Block -> tile of bwd_main: die x (blocks x, x + 8, ...) first runs its contiguous share of the locality-ordered tiles,
// then every 8th of the remaining ones; without an order the tiles run in index order.  -1: the block has no tile.
__device__ __forceinline__ int bwd_tile_of_block(int b, int num_tiles, const int32_t* __restrict__ order,
                                                 const int32_t* __restrict__ order_offsets) {
    const int nh = order ? order_offsets[kOrderBuckets] : 0;
    const int nc = num_tiles - nh;
    const int hc = (nh + kNumXcd - 1) / kNumXcd;
    const int x = b % kNumXcd, sl = b / kNumXcd;
    int k;
    if (!NP_ORDER_XCD_SPLIT) {
        k = b;
        if (k >= num_tiles) return -1;
    } else if (sl < hc) {
        k = x * hc + sl;
        if (k >= nh) return -1;
    } else {
        const int kc = (sl - hc) * kNumXcd + x;
        if (kc >= nc) return -1;
        k = nh + kc;
    }
    return order ? order[k] : k;
}

// Row index (tunable "bwd_row_index"): the upstream-gradient row (and the mean-pooling weight) of every sorted position,
// resolved once and laid out in the order in which bwd_main's blocks run: block b finds the rows of its 256 positions at
// srow[256 b ..] with one coalesced load that depends on nothing, and can request its first rows while it is still
// finding out which tile it has and where the segments lie.  -1 marks a position past the end.  Every thread resolves
// kRowsSlots positions at once (all loads unconditional, from clamped positions, so that the chains overlap).
constexpr int kRowsSlots = 8;

template <bool MEAN>
__global__ void __launch_bounds__(256)
bwd_rows_kernel(const int32_t* __restrict__ occ, int n, const BagMapEntry* __restrict__ map, const int32_t* __restrict__ bag_offsets,
                int seq, int max_len, int num_tiles, const int32_t* __restrict__ order, const int32_t* __restrict__ order_offsets,
                const int32_t* __restrict__ tile_seg0, int num_slots, int32_t* __restrict__ srow, float* __restrict__ sweight,
                int2* __restrict__ slot_info) {
    const int t = threadIdx.x;
    int tile[kRowsSlots], j[kRowsSlots];
    bool ok[kRowsSlots];
    // lane q of every wave maps slot q (block-uniform code, one slot after the other, would be eight dependent scalar
    // loads in a row), then the wave shares the eight tiles.  The kernel's time (0.36 ms for 42 M positions) is that of
    // its 42 M reads of 16 bytes scattered over the 10 MB bag map: the rate at which L2 misses of single lines are served.
    int my_tile = -1;
    {
        const int q = __lane_id() % kRowsSlots;
        const int s = blockIdx.x * kRowsSlots + q;
        if (s < num_slots) my_tile = bwd_tile_of_block(s, num_tiles, order, order_offsets);
    }
#pragma unroll
    for (int q = 0; q < kRowsSlots; ++q) tile[q] = __shfl(my_tile, q, kWave);
#pragma unroll
    for (int q = 0; q < kRowsSlots; ++q) {
        const int64_t i = static_cast<int64_t>(tile[q]) * kBwdTile + t;
        ok[q] = tile[q] >= 0 && i < n;
        j[q] = occ[ok[q] ? i : 0];
    }
    BagMapEntry e[kRowsSlots];
#pragma unroll
    for (int q = 0; q < kRowsSlots; ++q) e[q] = map[j[q] >> 6];
#pragma unroll
    for (int q = 0; q < kRowsSlots; ++q) {
        const int s = blockIdx.x * kRowsSlots + q;
        if (s >= num_slots) continue;
        int bag, start;
        bag_from_entry(e[q], bag_offsets, j[q], bag, start);
        const int64_t at = static_cast<int64_t>(s) * kBwdTile + t;
        srow[at] = ok[q] ? (seq ? bag * max_len + (j[q] - start) : bag) : -1;
        if (MEAN) sweight[at] = ok[q] ? 1.f / static_cast<float>(bag_offsets[bag + 1] - start) : 0.f;
        if (t == 0) slot_info[s] = make_int2(tile[q], tile[q] >= 0 ? tile_seg0[tile[q]] : 0);  // the block's tile and its first segment
    }
}

// Partition policy that sorts tiles by the bucket of their relative position inside a long segment; tiles that are
// not wholly inside one long segment go to the last bucket.
struct TileOrderPolicy {
    using KeyT = uint32_t;
    static constexpr bool kStageDigit = false;
    const int32_t* tile_seg0;
    const int32_t* occ_offsets;
    int32_t* order;
    int n;
    __device__ __forceinline__ uint32_t load_key(int64_t i) const {
        const int tile_start = static_cast<int>(i) * kBwdTile;
        const int tile_end = n - tile_start < kBwdTile ? n : tile_start + kBwdTile;
        const int u0 = tile_seg0[i];
        const int s0 = occ_offsets[u0], e0 = occ_offsets[u0 + 1];
        if (e0 < tile_end || e0 - s0 < kOrderMinCount) return kOrderBuckets;
        return static_cast<uint32_t>((static_cast<uint64_t>(tile_start - s0) * kOrderBuckets) / static_cast<uint32_t>(e0 - s0));
    }
    __device__ __forceinline__ void load(int64_t i, uint32_t& k, uint32_t& v) const {
        k = load_key(i);
        v = static_cast<uint32_t>(i);
    }
    __device__ __forceinline__ uint32_t digit(uint32_t k) const { return k; }
    __device__ __forceinline__ void store(uint32_t dst, uint32_t, uint32_t v) const { order[dst] = static_cast<int32_t>(v); }
    __device__ __forceinline__ void placed(int64_t, uint32_t) const {}
};

template <int LPR>
__device__ __forceinline__ int group_bcast(int v, int src_in_group) {
    return __shfl(v, (__lane_id() & ~(LPR - 1)) + src_in_group, kWave);
}

// Row `row` (non-negative, below 2^31) of dY: one 32x32->64 multiply for the byte offset.
__device__ __forceinline__ float4 load_dy(const float* dY, int row, int dim, int word) {
    const uint64_t off = static_cast<uint64_t>(static_cast<uint32_t>(row)) * static_cast<uint32_t>(dim * 4);
    return reinterpret_cast<const float4*>(reinterpret_cast<const char*>(dY) + off)[word];
}

__device__ __forceinline__ float4 load_dy(const uint16_t* dY, int row, int dim, int word) {
    const uint64_t off = static_cast<uint64_t>(static_cast<uint32_t>(row)) * static_cast<uint32_t>(dim * 2);
    const uint2 p = reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(dY) + off)[word];
    return make_float4(__uint_as_float(p.x << 16), __uint_as_float(p.x & 0xFFFF0000u), __uint_as_float(p.y << 16),
                       __uint_as_float(p.y & 0xFFFF0000u));
}

// Words 2 * pair and 2 * pair + 1 of a bf16 row with one 16-byte load (rows a multiple of 8 elements wide, 16-byte
// aligned base).  Twice the bytes per load instruction: with 8-byte lanes the gather of 256-byte bf16 rows in
// sequence mode ran at half the rate of the fp32 one.
__device__ __forceinline__ void load_dy_pair(const uint16_t* dY, int row, int dim, int pair, float4& a, float4& b) {
    const uint64_t off = static_cast<uint64_t>(static_cast<uint32_t>(row)) * static_cast<uint32_t>(dim * 2);
    const uint4 p = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(dY) + off)[pair];
    a = make_float4(__uint_as_float(p.x << 16), __uint_as_float(p.x & 0xFFFF0000u), __uint_as_float(p.y << 16),
                    __uint_as_float(p.y & 0xFFFF0000u));
    b = make_float4(__uint_as_float(p.z << 16), __uint_as_float(p.z & 0xFFFF0000u), __uint_as_float(p.w << 16),
                    __uint_as_float(p.w & 0xFFFF0000u));
}
__device__ __forceinline__ void load_dy_pair(const float*, int, int, int, float4&, float4&) {}  // never selected

// Variant (tunable "bwd_singles_by_bag", pooled modes, fp32 upstream gradients, plain sink): a key with ONE lookup needs no
// reduction, its gradient row is a copy of its bag's upstream row.  Such keys are served bag by bag, each upstream row
// read once and in order, instead of being gathered one row per key in key order; bwd_main then skips them.
//   bwd_single_fill   sdst[j] = -1 for every lookup
//   bwd_single_mark   for every key with one lookup j: sdst[j] = the row of grads it owns
//   bwd_single_copy   one LPR-lane group per bag: reads the bag's slice of sdst, and if any entry is set the bag's upstream
//                     row once; writes it (0 + x, or w * x for mean pooling: the operations of the key-major walk, so the
//                     bits are the same) to every set entry's row
__global__ void __launch_bounds__(256)
bwd_single_fill_kernel(int32_t* __restrict__ sdst, int n) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * 256) sdst[i] = -1;
}

__global__ void __launch_bounds__(256)
bwd_single_mark_kernel(const int32_t* __restrict__ occ_offsets, const int32_t* __restrict__ occ, const int32_t* __restrict__ d_num_unique,
                       int ucap, const int32_t* __restrict__ unique_to_send, int32_t* __restrict__ sdst) {
    const int U = device_count(d_num_unique, ucap);
    for (int64_t u = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; u < U; u += static_cast<int64_t>(gridDim.x) * 256) {
        const int a = occ_offsets[u];
        if (occ_offsets[u + 1] - a == 1) sdst[occ[a]] = unique_to_send ? unique_to_send[u] : static_cast<int32_t>(u);
    }
}

template <int LPR, int NV, bool MEAN>
__global__ void __launch_bounds__(256)
bwd_single_copy_kernel(const float* __restrict__ dY, int dim, const int32_t* __restrict__ bag_offsets, int num_bags,
                       const int32_t* __restrict__ sdst, float* __restrict__ grads) {
    constexpr int GPB = 256 / LPR;
    const int r = threadIdx.x % LPR;
    const int64_t b = static_cast<int64_t>(blockIdx.x) * GPB + threadIdx.x / LPR;
    if (b >= num_bags) return;  // whole groups leave together
    const int lo = bag_offsets[b], hi = bag_offsets[b + 1];
    const int words = dim / 4;
    const int gl = __lane_id() & ~(LPR - 1);
    const uint64_t gmask = (LPR == 64 ? ~0ull : ((1ull << (LPR & 63)) - 1ull)) << gl;
    float w = 1.f;
    if (MEAN && hi > lo) w = 1.f / static_cast<float>(hi - lo);
    bool have = false;
    float4 x[NV];
    for (int base = lo; base < hi; base += LPR) {
        const int j = base + r;
        const int mine = j < hi ? load_stream(sdst + j) : -1;
        uint64_t set = __ballot(mine >= 0) & gmask;
        if (set && !have) {  // uniform inside the group
            have = true;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int wv = r + v * LPR;
                float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                if (wv < words) t = load_dy(dY, static_cast<int>(b), dim, wv);
                // the first (and only) step of the key-major running sum
                if (MEAN) x[v] = make_float4(fmaf(w, t.x, 0.f), fmaf(w, t.y, 0.f), fmaf(w, t.z, 0.f), fmaf(w, t.w, 0.f));
                else x[v] = make_float4(0.f + t.x, 0.f + t.y, 0.f + t.z, 0.f + t.w);
            }
        }
        while (set) {
            const int lane = __builtin_ctzll(set);
            set &= set - 1;
            const int dst = __shfl(mine, lane, kWave);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int wv = r + v * LPR;
                if (wv < words) store_stream(reinterpret_cast<float4*>(grads + static_cast<size_t>(dst) * dim) + wv, x[v]);
            }
        }
    }
}

// Where a finished gradient row goes.  Plain (FUSED == 0): grads[dst, :].  Fused (np_lookup_bwd_adagrad): the row is
// consumed on the spot by the row-wise Adagrad step on table[keys[dst], :] and never reaches HBM; the arithmetic is
// the one of np_sparse_adagrad (same butterfly over the LPR lanes of a row, same store rounding), so both routes
// give the same bits.  FUSED also names the table's element type: 1 fp32, 2 bf16, 3 fp16.
constexpr int kSinkGrads = 0, kSinkF32 = 1, kSinkBf16 = 2, kSinkF16 = 3;

template <int FUSED> struct SinkTable { using type = float; };
template <> struct SinkTable<kSinkBf16> { using type = uint16_t; };
template <> struct SinkTable<kSinkF16> { using type = __half; };

struct RowSink {
    float* grads;
    void* table;
    float* state;
    const int64_t* keys;
    float lr, eps, inv_dim;
};

// The fused step once its operands are in registers: the key, the old state and the table row (lane r holds words
// r, r + LPR, ... in w[0 .. NV-1], zero past the row's end).  The arithmetic is that of np_sparse_adagrad's kernel,
// operation by operation (squares summed over the lane's words in ascending v, then the butterfly over the LPR lanes),
// so both routes give the same bits.
template <int LPR, int NV, int FUSED>
__device__ __forceinline__ void sink_row_loaded(const RowSink& sk, int64_t key, float s_old, int dim, int r, int words, float4 (&w)[NV],
                                                const float4 (&g)[NV]) {
    using TabT = typename SinkTable<FUSED>::type;
    TabT* wrow = static_cast<TabT*>(sk.table) + static_cast<size_t>(key) * dim;
    float ss = 0.f;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int wv = r + v * LPR;
        float4 gv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (wv < words) gv = g[v];
        ss += sumsq4(gv);
    }
#pragma unroll
    for (int d = LPR / 2; d > 0; d >>= 1) ss += __shfl_xor(ss, d, kWave);
    const float G = adagrad_state(s_old, ss, sk.inv_dim);
    const float denom = sqrtf(G) + sk.eps;
    if (r == 0) sk.state[key] = G;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int wv = r + v * LPR;
        if (wv < words) {
            adagrad_step4(w[v], g[v], sk.lr, denom);
            store_word_stream(wrow, wv, w[v]);
        }
    }
}

// Called by all LPR lanes that hold a row: lane r holds the float4 words r, r + LPR, ... in g[0 .. NV-1].
template <int LPR, int NV, int FUSED>
__device__ __forceinline__ void sink_row(const RowSink& sk, int dst, int dim, int r, int words, const float4 (&g)[NV]) {
    if constexpr (FUSED == kSinkGrads) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int wv = r + v * LPR;
            if (wv < words) store_stream(reinterpret_cast<float4*>(sk.grads + static_cast<size_t>(dst) * dim) + wv, g[v]);
        }
    } else {
        using TabT = typename SinkTable<FUSED>::type;
        const int64_t key = sk.keys[dst];
        const TabT* wrow = static_cast<const TabT*>(sk.table) + static_cast<size_t>(key) * dim;
        float4 w[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int wv = r + v * LPR;
            w[v] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (wv < words) w[v] = load_word(wrow, wv);
        }
        const float s_old = sk.state[key];
        sink_row_loaded<LPR, NV, FUSED>(sk, key, s_old, dim, r, words, w, g);
    }
}

// Which float4 word of the row lane r of a group holds in its v-th accumulator.  Striped (word r + v * LPR) by default;
// PAIR (NV == 2, bf16 dY): words 2r and 2r + 1, the 16 bytes of one bf16 load.  Everything past the walk (partials in
// LDS and in the workspace, the fix-up kernels) is indexed by word, so the layout is private to the walk.
template <int LPR, bool PAIR>
__device__ __forceinline__ int word_of(int r, int v) {
    return PAIR ? 2 * r + v : r + v * LPR;
}

template <int LPR, int NV, bool MEAN, typename DyT, int FUSED, bool PAIR = false>
__global__ void __launch_bounds__(256)
bwd_main_kernel(const DyT* __restrict__ dY, int dim, int seq, int max_len, const int32_t* __restrict__ bag_offsets, int n,
                const int32_t* __restrict__ occ_offsets, const int32_t* __restrict__ occ, const int32_t* __restrict__ d_num_unique,
                const int32_t* __restrict__ unique_to_send, const BagMapEntry* __restrict__ bagmap,
                const int32_t* __restrict__ tile_seg0, const int32_t* __restrict__ order, const int32_t* __restrict__ order_offsets,
                int num_tiles, int ucap, RowSink sink, float* __restrict__ tile_left, float* __restrict__ tile_right,
                int32_t* __restrict__ tile_rseg, const int32_t* __restrict__ srow, const float* __restrict__ sweight,
                const int2* __restrict__ slot_info, int skip_singles) {
    static_assert(!PAIR || (NV == 2 && FUSED == kSinkGrads), "the pair layout is two words per lane, plain sink");
    constexpr int GPB = 256 / LPR;
    constexpr int ROWW = LPR * NV;  // float4 words per (padded) row
    __shared__ int headmark[kBwdTile + 1];
    __shared__ int wave_heads[4];
    __shared__ float4 lpart[GPB * ROWW];
    __shared__ float4 rpart[GPB * ROWW];
    __shared__ int l_exists[GPB], l_closed[GPB], l_dst[GPB], r_exists[GPB];

    const int t = threadIdx.x;
    const int words = dim / 4;
    const int g = t / LPR, r = t % LPR;
    const int wv_id = t / kWave;
    // With the row index (srow, laid out block by block) the rows of this block's positions are known before the block
    // even knows its tile: the first batch of row loads goes out at once and is in flight while the tile, its segments
    // and the destinations are being found.
    const bool indexed = srow != nullptr;
    int sr = -1;
    float w = 1.f;
    int tile, u0;
    if (indexed) {
        sr = load_stream(srow + static_cast<int64_t>(blockIdx.x) * kBwdTile + t);
        if (MEAN) w = load_stream(sweight + static_cast<int64_t>(blockIdx.x) * kBwdTile + t);
        const int2 info = slot_info[blockIdx.x];
        tile = info.x;
        u0 = info.y;
    } else {
        tile = bwd_tile_of_block(blockIdx.x, num_tiles, order, order_offsets);
        u0 = tile >= 0 ? tile_seg0[tile] : 0;
    }
    if (tile < 0) return;  // uniform
    const int tile_start = tile * kBwdTile;
    const int i = tile_start + t;
    const bool valid = i < n;
    const int U = device_count(d_num_unique, ucap);  // ucap = min(n, cap): rows of grads / entries of unique_to_send
    if (u0 >= U) u0 = U > 0 ? U - 1 : 0;  // only with a count above the caller's bound (a broken precondition): stay inside the lists
    // The segment boundaries are requested BEFORE the rows: loads come back in the order they were issued, so what is
    // needed first has to be asked for first (unconditional, from a clamped index: occ_offsets[U] exists).
    const int cand = u0 + 1 + t;
    const int rel_raw = occ_offsets[cand <= U ? cand : U] - tile_start;
    const int seg0_start = occ_offsets[u0];
    const int j = (valid && !indexed) ? load_stream(occ + i) : 0;
    float4 x[kBwdUnroll][NV];
    // rows of positions k0 .. k0 + kBwdUnroll - 1 of the strip; a position without a row (sr < 0) or past `limit` loads nothing
    auto load_batch = [&](int k0, int limit) {
#pragma unroll
        for (int q = 0; q < kBwdUnroll; ++q) {
            const int srk = group_bcast<LPR>(sr, (k0 + q) & (LPR - 1));
            const bool on = k0 + q < limit && srk >= 0;
            if constexpr (PAIR) {
                x[q][0] = x[q][1] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (on && 2 * r < words) load_dy_pair(dY, srk, dim, r, x[q][0], x[q][1]);  // words is even here
            } else {
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int wv = r + v * LPR;
                    x[q][v] = (on && wv < words) ? load_dy(dY, srk, dim, wv) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
    };
    const bool early = indexed && !skip_singles;  // (the single-lookup variant decides later which rows it does not want)
    if (early) load_batch(0, LPR);
    const int rel = cand <= U ? rel_raw : INT32_MAX;  // >= 1
    // (the three barriers of this prologue order LDS traffic only: lds_barrier leaves the row loads in flight)
    headmark[t] = 0;
    if (t == 0) headmark[kBwdTile] = 0;
    lds_barrier();
    if (rel <= kBwdTile) headmark[rel] = 1;
    if (!indexed && valid) {
        int bag, start;
        bag_of_lookup(bagmap, bag_offsets, j, bag, start);
        sr = seq ? bag * max_len + (j - start) : bag;
        if (MEAN) w = 1.f / static_cast<float>(bag_offsets[bag + 1] - start);
    }
    lds_barrier();
    // segment of every position: heads strictly after the tile start, counted with one ballot per wave
    const int flag = t > 0 ? headmark[t] : 0;
    const int is_tail = headmark[t + 1];
    const uint64_t fmask = __ballot(flag);
    if (__lane_id() == 0) wave_heads[wv_id] = __popcll(fmask);
    lds_barrier();
    int seg = u0 + __popcll(fmask & lanemask_lt()) + flag;
#pragma unroll
    for (int ww = 0; ww < 3; ++ww)
        if (ww < wv_id) seg += wave_heads[ww];
    // a tail position knows where its segment's row goes; every other position carries -1
    int dst = -1;
    if (valid && is_tail) dst = unique_to_send ? unique_to_send[seg] : seg;
    if (valid && t == min(n - tile_start, kBwdTile) - 1) {
        // the tile owns the segment that runs past its end only if that segment starts inside the tile
        const bool starts_here = seg > u0 || seg0_start == tile_start;
        const bool owns = !is_tail && starts_here;
        // -1: the tile owns no cut segment; seg >= 0: a chain of up to kFixupShort left partials follows (summed by one
        // group); -2 - seg: a longer chain (summed by a whole block)
        int code = -1;
        if (owns) code = (occ_offsets[seg + 1] - 1) / kBwdTile - tile > kFixupShort ? -2 - seg : seg;
        tile_rseg[tile] = code;
    }

    if (skip_singles && valid && is_tail && (t == 0 ? seg0_start == tile_start : flag != 0)) {
        // a key with one lookup, served by the bag-major copy: no row to load here (sr < 0), nothing to store (-2: the
        // position closes nothing and leaves nothing open)
        sr = -1;
        dst = -2;
    }
    // Fused sink, rows of up to LPR words: what the Adagrad step of a finished row needs is requested ahead, so that no
    // group waits inside the walk for loads that depend on each other.  Every tail position fetches its key and the old
    // state here; the table rows travel with the dY rows of the batch they end in (load_table_batch).  A row's key, state
    // and table row are touched by exactly one sink per launch, so reading them early reads the same values.
    constexpr bool kSinkAhead = FUSED != kSinkGrads && NV == 1;
    int skey_lo = 0, skey_hi = 0;
    float sold = 0.f;
    if constexpr (kSinkAhead) {
        if (dst >= 0) {
            const int64_t key = sink.keys[dst];
            skey_lo = static_cast<int>(static_cast<uint32_t>(static_cast<uint64_t>(key)));
            skey_hi = static_cast<int>(static_cast<uint64_t>(key) >> 32);
            sold = sink.state[key];
        }
    }
    // the first position of the strip that ends a segment (LPR: none does)
    int first_tail = LPR;
    {
        const uint64_t tails = __ballot(dst >= 0) >> (__lane_id() & ~(LPR - 1) & (kWave - 1));
        const uint64_t mine = LPR == kWave ? tails : tails & ((1ull << (LPR & 63)) - 1);
        if (mine) first_tail = __builtin_ctzll(mine);
    }
    // ---- each group walks its strip of LPR positions ---------------------------------------------------
    // Position k > 0 starts a segment exactly when position k - 1 ends one, so the walk needs the end marks
    // (dst >= 0) and, for position 0 alone, whether the strip begins inside a segment that started earlier.
    int cnt = n - (tile_start + g * LPR);
    cnt = cnt < 0 ? 0 : (cnt > LPR ? LPR : cnt);
    const int head_here = t == 0 ? (seg0_start == tile_start ? 1 : 0) : flag;
    // Everything the walk has to decide is known per group before it starts: whether the strip's first run continues an
    // earlier one (then the first segment end closes a cut run: its sum is parked, not stored), and whether the last
    // position leaves a run open.  The loop carries the running sum and nothing else.
    const bool first_cut = group_bcast<LPR>(head_here, 0) == 0;
    const bool open_after = cnt > 0 && group_bcast<LPR>(dst, cnt > 0 ? cnt - 1 : 0) == -1;  // (-2, a skipped single-lookup key, leaves nothing open)
    const int wbits = __float_as_int(w);
    float4 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 tw[kSinkAhead ? kBwdUnroll : 1][NV];
    using TabT = typename SinkTable<FUSED>::type;
    // table rows of the tails among positions k0 .. k0 + kBwdUnroll - 1 that are finished inside this walk
    auto load_table_batch = [&](int k0) {
        if constexpr (kSinkAhead) {
#pragma unroll
            for (int q = 0; q < kBwdUnroll; ++q) {
                const int kk = (k0 + q) & (LPR - 1);
                const int dkq = group_bcast<LPR>(dst, kk);
                const int64_t key = static_cast<int64_t>((static_cast<uint64_t>(static_cast<uint32_t>(group_bcast<LPR>(skey_hi, kk))) << 32) |
                                                         static_cast<uint32_t>(group_bcast<LPR>(skey_lo, kk)));
                const bool need = k0 + q < cnt && dkq >= 0 && !(first_cut && k0 + q == first_tail) && r < words;
                const TabT* wrow = static_cast<const TabT*>(sink.table) + static_cast<size_t>(key) * dim;
                tw[q][0] = need ? load_word(wrow, r) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    for (int k0 = 0; k0 < cnt; k0 += kBwdUnroll) {
        if (!(early && k0 == 0)) load_batch(k0, cnt);
        load_table_batch(k0);
        // One explicit wait for the batch, outside every condition.  The loads above sit in conditional blocks, so without it
        // the compiler waits for "all outstanding memory operations" at every position that uses a loaded row, and after
        // a row has been stored that includes the store: every finished row would cost a round trip to memory.
        wait_vmem_all();
#pragma unroll
        for (int q = 0; q < kBwdUnroll; ++q) {
            const int k = k0 + q;
            if (k < cnt) {
                const int dk = group_bcast<LPR>(dst, k);
                const float wk = MEAN ? __int_as_float(group_bcast<LPR>(wbits, k)) : 1.f;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    if (MEAN) {
                        acc[v].x = fmaf(wk, x[q][v].x, acc[v].x);
                        acc[v].y = fmaf(wk, x[q][v].y, acc[v].y);
                        acc[v].z = fmaf(wk, x[q][v].z, acc[v].z);
                        acc[v].w = fmaf(wk, x[q][v].w, acc[v].w);
                    } else {
                        acc[v].x += x[q][v].x;
                        acc[v].y += x[q][v].y;
                        acc[v].z += x[q][v].z;
                        acc[v].w += x[q][v].w;
                    }
                }
                if (dk >= 0) {  // a segment ends here
                    if (!(first_cut && k == first_tail)) {
                        if constexpr (PAIR) {
#pragma unroll
                            for (int v = 0; v < NV; ++v) {
                                const int wv = word_of<LPR, PAIR>(r, v);
                                if (wv < words) store_stream(reinterpret_cast<float4*>(sink.grads + static_cast<size_t>(dk) * dim) + wv, acc[v]);
                            }
                        } else if constexpr (kSinkAhead) {
                            const int64_t key = static_cast<int64_t>((static_cast<uint64_t>(static_cast<uint32_t>(group_bcast<LPR>(skey_hi, k))) << 32) |
                                                                     static_cast<uint32_t>(group_bcast<LPR>(skey_lo, k)));
                            const float so = __int_as_float(group_bcast<LPR>(__float_as_int(sold), k));
                            sink_row_loaded<LPR, NV, FUSED>(sink, key, so, dim, r, words, tw[q], acc);
                        } else {
                            sink_row<LPR, NV, FUSED>(sink, dk, dim, r, words, acc);
                        }
                    } else {
#pragma unroll
                        for (int v = 0; v < NV; ++v) lpart[g * ROWW + word_of<LPR, PAIR>(r, v)] = acc[v];
                    }
#pragma unroll
                    for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
    }
    // what the strip hands to the combine stage
    const bool has_tail = first_tail < cnt;
    const bool le = first_cut && cnt > 0 && (has_tail || open_after);  // a run that began before the strip ...
    const bool lc = first_cut && has_tail;                               // ... and ends inside it
    const int ld = lc ? group_bcast<LPR>(dst, first_tail & (LPR - 1)) : -1;
    const bool whole = first_cut && !has_tail && open_after;             // one run covers the whole strip
    const bool re = open_after && !whole;                                // a run that starts in the strip and goes on
    if (whole) {
#pragma unroll
        for (int v = 0; v < NV; ++v) lpart[g * ROWW + word_of<LPR, PAIR>(r, v)] = acc[v];
    } else if (re) {
#pragma unroll
        for (int v = 0; v < NV; ++v) rpart[g * ROWW + word_of<LPR, PAIR>(r, v)] = acc[v];
    }
    if (r == 0) {
        l_exists[g] = le;
        l_closed[g] = lc;
        l_dst[g] = ld;
        r_exists[g] = re;
    }
    __syncthreads();

    // ---- combine the cut sums across the groups, in strip order; thread c < LPR owns words c, c + LPR, ... of the row ----
    if (t < LPR) {
        float4 carry[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) carry[v] = make_float4(0.f, 0.f, 0.f, 0.f);
        bool open = false, started_here = false;
        for (int gg = 0; gg < GPB; ++gg) {
            if (l_exists[gg]) {
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const float4 p = lpart[gg * ROWW + t + v * LPR];
                    if (open) {
                        carry[v].x += p.x;
                        carry[v].y += p.y;
                        carry[v].z += p.z;
                        carry[v].w += p.w;
                    } else {
                        carry[v] = p;
                    }
                }
                if (!open) {
                    started_here = false;
                    open = true;
                }
                if (l_closed[gg]) {
                    if (started_here) {
                        sink_row<LPR, NV, FUSED>(sink, l_dst[gg], dim, t, words, carry);
                    } else {
#pragma unroll
                        for (int v = 0; v < NV; ++v)
                            if (t + v * LPR < words) reinterpret_cast<float4*>(tile_left + static_cast<size_t>(tile) * dim)[t + v * LPR] = carry[v];
                    }
                    open = false;
                }
            }
            if (r_exists[gg]) {
#pragma unroll
                for (int v = 0; v < NV; ++v) carry[v] = rpart[gg * ROWW + t + v * LPR];
                open = true;
                started_here = true;
            }
        }
        if (open) {
            float* side = started_here ? tile_right : tile_left;
#pragma unroll
            for (int v = 0; v < NV; ++v)
                if (t + v * LPR < words) reinterpret_cast<float4*>(side + static_cast<size_t>(tile) * dim)[t + v * LPR] = carry[v];
        }
    }
}

// A tile whose last segment runs on into later tiles owns that segment: it adds its right partial and the left
// partials of the following tiles, in tile order.  Chains of up to kFixupShort partials (nearly all of them) are
// summed by one LPR-lane group per tile; longer chains (a key with millions of lookups spans thousands of tiles)
// are listed and summed by a whole block each, cut into one contiguous run per group with four loads in
// flight per lane.  Either way the shape of the sum depends on the chain length alone.
constexpr int kFixupThreads = 1024;
constexpr int kFixupLongBlocks = 512;  // blocks that walk the list of long chains

template <int LPR, int NV, int FUSED>
__device__ __forceinline__ void fixup_short_part(int first_block_tile, int dim, int num_tiles, const int32_t* __restrict__ occ_offsets,
                                                 const int32_t* __restrict__ unique_to_send, const float* __restrict__ tile_left,
                                                 const float* __restrict__ tile_right, const int32_t* __restrict__ tile_rseg,
                                                 const RowSink& sink) {
    const int r = threadIdx.x % LPR;
    const int tile = first_block_tile + threadIdx.x / LPR;
    if (tile >= num_tiles) return;
    const int seg = tile_rseg[tile];
    if (seg < 0) return;
    const int count = (occ_offsets[seg + 1] - 1) / kBwdTile - tile;  // left partials to add, 1..kFixupShort (longer chains carry a code < -1)
    const int words = dim / 4;
    float4 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int wv = r + v * LPR;
        acc[v] = wv < words ? reinterpret_cast<const float4*>(tile_right + static_cast<size_t>(tile) * dim)[wv]
                            : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int c = 0; c < count; ++c) {
        const float4* src = reinterpret_cast<const float4*>(tile_left + static_cast<size_t>(tile + 1 + c) * dim);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int wv = r + v * LPR;
            if (wv < words) {
                const float4 p = src[wv];
                acc[v].x += p.x;
                acc[v].y += p.y;
                acc[v].z += p.z;
                acc[v].w += p.w;
            }
        }
    }
    const int dst = unique_to_send ? unique_to_send[seg] : seg;
    sink_row<LPR, NV, FUSED>(sink, dst, dim, r, words, acc);
}

// One launch for both kinds of chain: the last short_blocks blocks take one tile per LPR-lane group (chains of up to
// kFixupShort partials), the blocks before them take the long chains, one chain per block at a time.
// Threads per block: 1024, or 512 for the widest rows (NV = 4), so that the block's partial rows stay within 32 KB of LDS.
template <int NV>
constexpr int fixup_threads() {
    return NV >= 4 ? kFixupThreads / 2 : kFixupThreads;
}

template <int LPR, int NV, int FUSED>
__global__ void __launch_bounds__(kFixupThreads)
bwd_fixup_kernel(int dim, int num_tiles, int short_blocks, const int32_t* __restrict__ occ_offsets,
                 const int32_t* __restrict__ unique_to_send, const float* __restrict__ tile_left, const float* __restrict__ tile_right,
                 const int32_t* __restrict__ tile_rseg, RowSink sink) {
    constexpr int FT = fixup_threads<NV>();
    constexpr int GPB = FT / LPR;
    constexpr int ROWW = LPR * NV;
    __shared__ float4 part[GPB * ROWW];
    // the blocks of the long chains come first in the grid: the longest chain is the critical path of the launch and
    // should start at once, the short chains fill the rest of the GPU beside it
    const int long_blocks = gridDim.x - short_blocks;
    if (static_cast<int>(blockIdx.x) >= long_blocks) {  // uniform per block
        fixup_short_part<LPR, NV, FUSED>((blockIdx.x - long_blocks) * GPB, dim, num_tiles, occ_offsets, unique_to_send, tile_left,
                                         tile_right, tile_rseg, sink);
        return;
    }
    // Long chains: block b of this part owns the tiles b, b + long_blocks, ...; every round all threads look at one owned
    // tile each, those that start a long chain are collected in LDS (in arbitrary order: it decides no value), then the
    // whole block sums the collected chains one after the other.
    __shared__ int found[FT];
    __shared__ int num_found;
    const int g = threadIdx.x / LPR, r = threadIdx.x % LPR;
    const int words = dim / 4;
    const int64_t round_span = static_cast<int64_t>(long_blocks) * FT;
    for (int64_t base = blockIdx.x; base < num_tiles; base += round_span) {
      __syncthreads();  // found[] and num_found of the previous round are no longer read
      if (threadIdx.x == 0) num_found = 0;
      __syncthreads();
      {
          const int64_t cand = base + static_cast<int64_t>(threadIdx.x) * long_blocks;
          if (cand < num_tiles && tile_rseg[cand] < -1) found[atomicAdd(&num_found, 1)] = static_cast<int>(cand);
      }
      __syncthreads();
      const int nf = num_found;
      for (int li = 0; li < nf; ++li) {
        const int tile = found[li];
        const int seg = -2 - tile_rseg[tile];
        const int count = (occ_offsets[seg + 1] - 1) / kBwdTile - tile;
        const int per = (count + GPB - 1) / GPB;
        const int c0 = g * per;
        const int c1 = c0 + per < count ? c0 + per : count;
        float4 acc[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);
        // the chain of the most popular key is the critical path of this kernel: many partial rows in flight per lane
        constexpr int kInFlight = 16 / NV;
        for (int c = c0; c < c1; c += kInFlight) {
            float4 p[kInFlight][NV];
#pragma unroll
            for (int q = 0; q < kInFlight; ++q) {
                const float4* src = reinterpret_cast<const float4*>(tile_left + static_cast<size_t>(tile + 1 + (c + q < c1 ? c + q : c)) * dim);
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int wv = r + v * LPR;
                    p[q][v] = (c + q < c1 && wv < words) ? src[wv] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
#pragma unroll
            for (int q = 0; q < kInFlight; ++q) {
                if (c + q < c1) {
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        acc[v].x += p[q][v].x;
                        acc[v].y += p[q][v].y;
                        acc[v].z += p[q][v].z;
                        acc[v].w += p[q][v].w;
                    }
                }
            }
        }
        __syncthreads();  // part may still be read for the previous chain of this block
#pragma unroll
        for (int v = 0; v < NV; ++v) part[g * ROWW + r + v * LPR] = acc[v];
        __syncthreads();
        const int t = threadIdx.x;
        if (t < LPR) {  // the first LPR threads hold NV words of the row each (words past the row are zeros)
            float4 sum[NV];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                sum[v] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (t + v * LPR < words) sum[v] = reinterpret_cast<const float4*>(tile_right + static_cast<size_t>(tile) * dim)[t + v * LPR];
            }
            for (int gg = 0; gg < GPB; ++gg) {
                if (gg * per < count) {
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const float4 q = part[gg * ROWW + t + v * LPR];
                        sum[v].x += q.x;
                        sum[v].y += q.y;
                        sum[v].z += q.z;
                        sum[v].w += q.w;
                    }
                }
            }
            const int dst = unique_to_send ? unique_to_send[seg] : seg;
            sink_row<LPR, NV, FUSED>(sink, dst, dim, t, words, sum);
        }
      }
    }
}

struct BwdWs {
    size_t total;
    int num_tiles;
};

// Blocks of bwd_main: one per tile, plus room for the dies' shares of the two kinds of tiles not being whole multiples.
inline size_t bwd_num_slots(int num_tiles) { return static_cast<size_t>((num_tiles + 2 * kNumXcd + kNumXcd - 1) / kNumXcd * kNumXcd); }

inline BwdWs bwd_ws_layout(int32_t n, int32_t dim, int32_t mode = NP_POOL_MEAN) {
    BwdWs w;
    w.num_tiles = (n + kBwdTile - 1) / kBwdTile;
    w.total = align_up(sizeof(BagMapEntry) * ((static_cast<size_t>(n) + 63) / 64), 256)  // bag map
              + 2 * align_up(4 * static_cast<size_t>(w.num_tiles) * dim, 256)        // tile_left, tile_right
              + 3 * align_up(4 * static_cast<size_t>(w.num_tiles), 256)              // tile_seg0, tile_rseg, order
              + align_up(4 * static_cast<size_t>(kOrderBuckets + 2), 256)             // bucket offsets of the order
              + align_up(4 * part_hist_elems(make_chunk_plan(w.num_tiles), kOrderBuckets + 1), 256)
              + align_up(4 * static_cast<size_t>(kOrderBuckets + 1), 256)
              + align_up(4 * bwd_num_slots(w.num_tiles) * kBwdTile, 256)                // row index per block and position
              + (mode == NP_POOL_MEAN ? align_up(4 * bwd_num_slots(w.num_tiles) * kBwdTile, 256) : 0)   // and its weight
              + align_up(8 * bwd_num_slots(w.num_tiles), 256)                             // tile and first segment of every block
              + (mode != NP_SEQ ? align_up(4 * static_cast<size_t>(n), 256) : 0);       // owner row of single-lookup keys (variant)
    return w;
}

struct BwdArgs {
    const void* dY;
    int dy_dtype, dim, mode, max_len;
    const int32_t* bag_offsets;
    int num_bags, n;
    const int32_t* occ_offsets;
    const int32_t* occ;
    const int32_t* d_num_unique;
    int cap;
    const int32_t* unique_to_send;
    RowSink sink;
    void* ws;
    hipStream_t stream;
    bool prepared;  // the workspace already holds what bwd_prepare_launch writes (np_lookup_bwd_prepare ran on it)
};

// Where everything lives in the caller's workspace, and whether the tile order is used.  A function of the sizes and
// modes alone, so the preparing call and the reducing call agree on it.
struct BwdPlan {
    BagMapEntry* bagmap;
    float* tile_left;
    float* tile_right;
    int32_t* tile_seg0;
    int32_t* tile_rseg;
    int32_t* order;
    int32_t* order_offsets;
    uint32_t* oH;
    uint32_t* obin;
    ChunkPlan oplan;
    int num_tiles, map_entries;
    bool ordered;
    int32_t* srow;   // "bwd_row_index": upstream-gradient row per block and position
    float* sweight;  // mean pooling only
    int2* slot_info;   // tile and first segment of every block
    int num_slots;
    int32_t* sdst;   // variant "bwd_singles_by_bag", pooled modes only
};

inline BwdPlan bwd_plan(const BwdArgs& a) {
    const BwdWs L = bwd_ws_layout(a.n, a.dim, a.mode);
    WsCursor cur(a.ws);
    BwdPlan P;
    P.num_tiles = L.num_tiles;
    P.map_entries = (a.n + 63) / 64;
    P.bagmap = cur.take<BagMapEntry>(P.map_entries);
    P.tile_left = cur.take<float>(static_cast<size_t>(L.num_tiles) * a.dim);
    P.tile_right = cur.take<float>(static_cast<size_t>(L.num_tiles) * a.dim);
    P.tile_seg0 = cur.take<int32_t>(L.num_tiles);
    P.tile_rseg = cur.take<int32_t>(L.num_tiles);
    P.order = cur.take<int32_t>(L.num_tiles);
    P.order_offsets = cur.take<int32_t>(kOrderBuckets + 2);
    P.oplan = make_chunk_plan(L.num_tiles);
    P.oH = cur.take<uint32_t>(part_hist_elems(P.oplan, kOrderBuckets + 1));
    P.obin = cur.take<uint32_t>(kOrderBuckets + 1);
    P.num_slots = static_cast<int>(bwd_num_slots(L.num_tiles));
    P.srow = cur.take<int32_t>(static_cast<size_t>(P.num_slots) * kBwdTile);
    P.sweight = a.mode == NP_POOL_MEAN ? cur.take<float>(static_cast<size_t>(P.num_slots) * kBwdTile) : nullptr;
    P.slot_info = cur.take<int2>(P.num_slots);
    P.sdst = a.mode != NP_SEQ ? cur.take<int32_t>(a.n) : nullptr;
    const bool seq = a.mode == NP_SEQ;
    // The locality order pays when dY is larger than the last-level cache (2.42 -> 2.06 ms at 1.3 GB); below that it only
    // costs three launches (0.63 -> 0.57 ms per step at 109 MB).  In sequence mode every dY row is read exactly once, so
    // there is nothing to share: the pass would cost more (0.04 ms) than the slightly friendlier read order returns
    // (0.02 ms on configuration 3).
    const size_t dy_bytes = static_cast<size_t>(a.num_bags) * (seq ? a.max_len : 1) * a.dim * (a.dy_dtype == NP_BF16 ? 2 : 4);
    P.ordered = static_cast<int64_t>(dy_bytes) > tune_get(kTuneBwdOrderMinDyBytes) && !seq;  // initially 256 MB, the Infinity Cache: a dY that fits it is re-read from there anyway
    return P;
}

// Everything that depends on the batch's index arrays alone (bag offsets, occurrence offsets), not on dY.
inline void bwd_prepare_launch(const BwdArgs& a, const BwdPlan& P) {
    const int map_blocks = (P.map_entries + 255) / 256, seg_blocks = (P.num_tiles + 255) / 256;
    NP_LAUNCH("bwd_prepare", bwd_prepare_kernel, dim3(map_blocks + seg_blocks), dim3(256), 0, a.stream, a.bag_offsets, a.num_bags,
              a.n, P.bagmap, map_blocks, a.occ_offsets, a.d_num_unique, P.num_tiles, P.tile_seg0);
    if (P.ordered) {
        TileOrderPolicy pol{P.tile_seg0, a.occ_offsets, P.order, a.n};
        run_partition_pass(pol, P.num_tiles, nullptr, kOrderBuckets + 1, 11, P.oplan, P.oH, P.obin, nullptr, P.order_offsets,
                           a.stream, "bwd_order_hist", "bwd_order_colscan", "bwd_order_scatter");
    }
    if (tune_get(kTuneBwdRowIndex) != 0) {
        const int32_t* order = P.ordered ? P.order : nullptr;
        const int32_t* order_offsets = P.ordered ? P.order_offsets : nullptr;
        const int g = (P.num_slots + kRowsSlots - 1) / kRowsSlots;
        if (a.mode == NP_POOL_MEAN)
            NP_LAUNCH("bwd_rows", bwd_rows_kernel<true>, dim3(g), dim3(256), 0, a.stream, a.occ, a.n, P.bagmap, a.bag_offsets, 0, a.max_len,
                      P.num_tiles, order, order_offsets, P.tile_seg0, P.num_slots, P.srow, P.sweight, P.slot_info);
        else
            NP_LAUNCH("bwd_rows", bwd_rows_kernel<false>, dim3(g), dim3(256), 0, a.stream, a.occ, a.n, P.bagmap, a.bag_offsets,
                      a.mode == NP_SEQ ? 1 : 0, a.max_len, P.num_tiles, order, order_offsets, P.tile_seg0, P.num_slots, P.srow,
                      P.sweight, P.slot_info);
    }
}

template <int LPR, int NV, int FUSED>
void bwd_launch(const BwdArgs& a) {
    const BwdPlan P = bwd_plan(a);
    if (!a.prepared) bwd_prepare_launch(a, P);
    const bool row_index = tune_get(kTuneBwdRowIndex) != 0;  // the preparing call wrote the index under the same setting
    const int32_t* srow = row_index ? P.srow : nullptr;
    const float* sweight = row_index ? P.sweight : nullptr;
    const int2* slot_info = row_index ? P.slot_info : nullptr;
    // single-lookup keys bag by bag: pooled modes, fp32 upstream gradients, gradient rows as the sink
    const bool singles = FUSED == kSinkGrads && a.mode != NP_SEQ && a.dy_dtype == NP_F32 && !a.prepared &&
                         tune_get(kTuneBwdSinglesByBag) != 0;
    if (singles) {
        int g = (a.n + 255) / 256;
        if (g > 16384) g = 16384;
        NP_LAUNCH("bwd_single_fill", bwd_single_fill_kernel, dim3(g), dim3(256), 0, a.stream, P.sdst, a.n);
        NP_LAUNCH("bwd_single_mark", bwd_single_mark_kernel, dim3(g), dim3(256), 0, a.stream, a.occ_offsets, a.occ, a.d_num_unique,
                  a.cap < a.n ? a.cap : a.n, a.unique_to_send, P.sdst);
        constexpr int GPB = 256 / LPR;
        const unsigned cg = static_cast<unsigned>((static_cast<int64_t>(a.num_bags) + GPB - 1) / GPB);
        if (a.mode == NP_POOL_MEAN)
            NP_LAUNCH("bwd_single_copy", (bwd_single_copy_kernel<LPR, NV, true>), dim3(cg), dim3(256), 0, a.stream,
                      static_cast<const float*>(a.dY), a.dim, a.bag_offsets, a.num_bags, P.sdst, a.sink.grads);
        else
            NP_LAUNCH("bwd_single_copy", (bwd_single_copy_kernel<LPR, NV, false>), dim3(cg), dim3(256), 0, a.stream,
                      static_cast<const float*>(a.dY), a.dim, a.bag_offsets, a.num_bags, P.sdst, a.sink.grads);
    }
    struct { int num_tiles; } L{P.num_tiles};
    BagMapEntry* bagmap = P.bagmap;
    float* tile_left = P.tile_left;
    float* tile_right = P.tile_right;
    int32_t* tile_seg0 = P.tile_seg0;
    int32_t* tile_rseg = P.tile_rseg;
    int32_t* order = P.ordered ? P.order : nullptr;  // no order: tiles run in index order
    int32_t* order_offsets = P.ordered ? P.order_offsets : nullptr;
    const int seq = a.mode == NP_SEQ ? 1 : 0;
    const unsigned main_grid = static_cast<unsigned>(P.num_slots);
    const bool mean = a.mode == NP_POOL_MEAN;
#define NP_BWD_MAIN(L_, N_, M_, T_, P_)                                                                                        \
    NP_LAUNCH("bwd_main", (bwd_main_kernel<L_, N_, M_, T_, FUSED, P_>), dim3(main_grid), dim3(256), 0, a.stream,                 \
              static_cast<const T_*>(a.dY), a.dim, seq, a.max_len, a.bag_offsets, a.n, a.occ_offsets, a.occ, a.d_num_unique,     \
              a.unique_to_send, bagmap, tile_seg0, order, order_offsets, L.num_tiles, a.cap < a.n ? a.cap : a.n, a.sink, tile_left, tile_right, tile_rseg, srow, sweight, slot_info, singles ? 1 : 0)
    bool launched = false;
    if constexpr (FUSED == kSinkGrads && NV == 1 && LPR >= 8) {
        // bf16 rows a multiple of 8 elements wide: half the lanes per row, 16-byte loads (words 2r, 2r + 1 per lane)
        if (a.dy_dtype == NP_BF16 && a.dim % 8 == 0 && aligned(a.dY, 16)) {
            if (mean) NP_BWD_MAIN(LPR / 2, 2, true, uint16_t, true);
            else NP_BWD_MAIN(LPR / 2, 2, false, uint16_t, true);
            launched = true;
        }
    }
    if (launched) {
    } else if (a.dy_dtype == NP_BF16) {
        if (mean) NP_BWD_MAIN(LPR, NV, true, uint16_t, false);
        else NP_BWD_MAIN(LPR, NV, false, uint16_t, false);
    } else {
        if (mean) NP_BWD_MAIN(LPR, NV, true, float, false);
        else NP_BWD_MAIN(LPR, NV, false, float, false);
    }
#undef NP_BWD_MAIN
    constexpr int kFixGPB = fixup_threads<NV>() / LPR;
    const int short_blocks = (L.num_tiles + kFixGPB - 1) / kFixGPB;
    NP_LAUNCH("bwd_fixup", (bwd_fixup_kernel<LPR, NV, FUSED>), dim3(short_blocks + kFixupLongBlocks), dim3(fixup_threads<NV>()), 0, a.stream,
              a.dim, L.num_tiles, short_blocks, a.occ_offsets, a.unique_to_send, tile_left, tile_right, tile_rseg, a.sink);
}

template <int FUSED>
void bwd_dispatch(const BwdArgs& a, int words) {
    if (words <= 4) bwd_launch<4, 1, FUSED>(a);
    else if (words <= 8) bwd_launch<8, 1, FUSED>(a);
    else if (words <= 16) bwd_launch<16, 1, FUSED>(a);
    else if (words <= 32) bwd_launch<32, 1, FUSED>(a);
    else if (words <= 64) bwd_launch<64, 1, FUSED>(a);
    else if (words <= 128) bwd_launch<64, 2, FUSED>(a);
    else bwd_launch<64, 4, FUSED>(a);
}

}  // namespace np

extern "C" {

size_t np_lookup_bwd_workspace_bytes(int32_t num_bags, int32_t n, int32_t dim, int32_t mode) {
    (void)num_bags;
    (void)mode;
    if (n <= 0 || dim < 4) return 0;
    return np::bwd_ws_layout(n, dim, mode).total;
}

// Argument checks shared by np_lookup_bwd_prepare (dY, occ and grads absent) and the reducing calls.
static int bwd_check_common(int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len, const int32_t* bag_offsets,
                            int32_t num_bags, int32_t n, const int32_t* occ_offsets, const int32_t* d_num_unique, int32_t dim_limit,
                            const void* ws, size_t ws_bytes, bool* nothing_to_do) {
    *nothing_to_do = false;
    if (num_bags < 0 || n < 0 || !d_num_unique) return NP_ERR_INVALID_ARG;
    if (mode != NP_POOL_SUM && mode != NP_POOL_MEAN && mode != NP_SEQ) return NP_ERR_INVALID_ARG;
    if (dy_dtype != NP_F32 && dy_dtype != NP_BF16) return NP_ERR_INVALID_ARG;
    if (mode == NP_SEQ && max_len < 1) return NP_ERR_INVALID_ARG;
    if (dim < 4 || dim % 4 != 0 || dim > dim_limit) return NP_ERR_UNSUPPORTED;
    if (mode == NP_SEQ && static_cast<int64_t>(num_bags) * max_len > INT32_MAX) return NP_ERR_UNSUPPORTED;
    if (n == 0) {  // no lookups: no key receives a gradient, nothing to write
        *nothing_to_do = true;
        return NP_OK;
    }
    if (n > INT32_MAX - (1 << 20)) return NP_ERR_UNSUPPORTED;  // tile-rounded positions must stay below 2^31
    if (!bag_offsets || !occ_offsets || num_bags < 1) return NP_ERR_INVALID_ARG;
    if (!ws || !np::aligned(ws, 256) || ws_bytes < np_lookup_bwd_workspace_bytes(num_bags, n, dim, mode)) return NP_ERR_WORKSPACE;
    return NP_OK;
}

int np_lookup_bwd_prepare(int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len, const int32_t* bag_offsets,
                          int32_t num_bags, int32_t n, const int32_t* occ_offsets, const int32_t* occ, const int32_t* d_num_unique,
                          void* ws, size_t ws_bytes, void* stream) {
    bool nothing = false;
    const int rc = bwd_check_common(dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, d_num_unique, NP_MAX_DIM, ws,
                                    ws_bytes, &nothing);
    if (rc != NP_OK || nothing) return rc;
    if (!occ) return NP_ERR_INVALID_ARG;
    np::BwdArgs a{nullptr, dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, occ, d_num_unique, n, nullptr,
                  np::RowSink{nullptr, nullptr, nullptr, nullptr, 0.f, 0.f, 0.f}, ws, static_cast<hipStream_t>(stream), false};
    np::bwd_prepare_launch(a, np::bwd_plan(a));
    return np::launch_status();
}

static int bwd_reduce(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len, const int32_t* bag_offsets,
                      int32_t num_bags, int32_t n, const int32_t* occ_offsets, const int32_t* occ, const int32_t* d_num_unique,
                      int32_t cap, const int32_t* unique_to_send, float* grads, void* ws, size_t ws_bytes, void* stream,
                      bool prepared) {
    if (cap < 0) return NP_ERR_INVALID_ARG;
    bool nothing = false;
    const int rc = bwd_check_common(dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, d_num_unique, NP_MAX_DIM, ws,
                                    ws_bytes, &nothing);
    if (rc != NP_OK || nothing) return rc;
    if (!dY || !occ || !grads) return NP_ERR_INVALID_ARG;
    if (!np::aligned(dY, dy_dtype == NP_BF16 ? 8 : 16) || !np::aligned(grads, 16)) return NP_ERR_INVALID_ARG;
    np::BwdArgs a{dY, dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, occ, d_num_unique, cap, unique_to_send,
                  np::RowSink{grads, nullptr, nullptr, nullptr, 0.f, 0.f, 0.f}, ws, static_cast<hipStream_t>(stream), prepared};
    np::bwd_dispatch<np::kSinkGrads>(a, dim / 4);
    return np::launch_status();
}

int np_lookup_bwd(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                  const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* occ_offsets,
                  const int32_t* occ, const int32_t* d_num_unique, int32_t cap, const int32_t* unique_to_send,
                  float* grads, void* ws, size_t ws_bytes, void* stream) {
    return bwd_reduce(dY, dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, occ, d_num_unique, cap, unique_to_send,
                      grads, ws, ws_bytes, stream, false);
}

int np_lookup_bwd_prepared(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                           const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* occ_offsets,
                           const int32_t* occ, const int32_t* d_num_unique, int32_t cap, const int32_t* unique_to_send,
                           float* grads, void* ws, size_t ws_bytes, void* stream) {
    return bwd_reduce(dY, dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, occ, d_num_unique, cap, unique_to_send,
                      grads, ws, ws_bytes, stream, true);
}

int np_lookup_bwd_adagrad_t(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                            const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* occ_offsets,
                            const int32_t* occ, const int64_t* unique, const int32_t* d_num_unique, int32_t cap, void* table,
                            int32_t table_dtype, float* state, int64_t num_rows, float lr, float eps, void* ws, size_t ws_bytes,
                            void* stream) {
    if (num_bags < 0 || n < 0 || cap < 0 || !d_num_unique || !table || !state || num_rows < 1) return NP_ERR_INVALID_ARG;
    if (table_dtype != NP_F32 && table_dtype != NP_BF16 && table_dtype != NP_F16) return NP_ERR_INVALID_ARG;
    if (mode != NP_POOL_SUM && mode != NP_POOL_MEAN && mode != NP_SEQ) return NP_ERR_INVALID_ARG;
    if (dy_dtype != NP_F32 && dy_dtype != NP_BF16) return NP_ERR_INVALID_ARG;
    if (mode == NP_SEQ && max_len < 1) return NP_ERR_INVALID_ARG;
    if (dim < 4 || dim % 4 != 0 || dim > NP_MAX_DIM) return NP_ERR_UNSUPPORTED;
    if (mode == NP_SEQ && static_cast<int64_t>(num_bags) * max_len > INT32_MAX) return NP_ERR_UNSUPPORTED;
    if (n == 0) return NP_OK;
    if (n > INT32_MAX - (1 << 20)) return NP_ERR_UNSUPPORTED;
    if (!dY || !bag_offsets || !occ_offsets || !occ || !unique || num_bags < 1) return NP_ERR_INVALID_ARG;
    if (!np::aligned(dY, dy_dtype == NP_BF16 ? 8 : 16) || !np::aligned(table, table_dtype == NP_F32 ? 16 : 8))
        return NP_ERR_INVALID_ARG;
    if (!ws || !np::aligned(ws, 256) || ws_bytes < np_lookup_bwd_workspace_bytes(num_bags, n, dim, mode)) return NP_ERR_WORKSPACE;
    np::BwdArgs a{dY, dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, occ, d_num_unique, cap, nullptr,
                  np::RowSink{nullptr, table, state, unique, lr, eps, 1.0f / static_cast<float>(dim)}, ws,
                  static_cast<hipStream_t>(stream), false};
    const int words = dim / 4;
    if (table_dtype == NP_BF16) np::bwd_dispatch<np::kSinkBf16>(a, words);
    else if (table_dtype == NP_F16) np::bwd_dispatch<np::kSinkF16>(a, words);
    else np::bwd_dispatch<np::kSinkF32>(a, words);
    return np::launch_status();
}

int np_lookup_bwd_adagrad(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                          const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* occ_offsets,
                          const int32_t* occ, const int64_t* unique, const int32_t* d_num_unique, int32_t cap, float* table,
                          float* state, int64_t num_rows, float lr, float eps, void* ws, size_t ws_bytes, void* stream) {
    return np_lookup_bwd_adagrad_t(dY, dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, occ, unique,
                                   d_num_unique, cap, table, NP_F32, state, num_rows, lr, eps, ws, ws_bytes, stream);
}

}  // extern "C"
