// np_dedup: distinct keys, inverse map, multiplicities and stable occurrence lists of a key batch
// (Section IV-A, "Key Routing": the sparse keys of a batch are deduplicated before anything is sent).
//
// Method: a stable LSD radix sort of (key, position) pairs over the low key_bits bits, then one pass
// over the sorted sequence that ranks the segment heads.  The sorted positions ARE the occurrence
// list; the rank of the segment a position falls in IS its inverse index.  Everything is a pure
// function of the input: no atomics decide an output value.
#include "np_partition.hpp"

namespace np {

#ifndef NP_MAX_DIGIT_BITS
#define NP_MAX_DIGIT_BITS 11
#endif
constexpr int kMaxDigitBits = NP_MAX_DIGIT_BITS;

struct PassPlan {
    int passes;
    int bits[8];
    int shift[8];
};

inline PassPlan make_pass_plan(int key_bits) {
    PassPlan p;
    p.passes = (key_bits + kMaxDigitBits - 1) / kMaxDigitBits;
    int left = key_bits, shift = 0;
    for (int i = 0; i < p.passes; ++i) {
        const int b = (left + (p.passes - i) - 1) / (p.passes - i);  // spread the bits evenly
        p.bits[i] = b;
        p.shift[i] = shift;
        shift += b;
        left -= b;
    }
    return p;
}

// First pass: items come straight from the int64 key array, the payload is the position.
template <typename K>
struct SortFirstPolicy {
    using KeyT = K;
    static constexpr bool kStageDigit = false;
    const int64_t* keys;
    K* out_k;
    uint32_t* out_v;
    int shift;
    uint32_t mask;
    __device__ __forceinline__ K load_key(int64_t i) const { return static_cast<K>(keys[i]); }
    __device__ __forceinline__ void load(int64_t i, K& k, uint32_t& v) const {
        k = static_cast<K>(keys[i]);
        v = static_cast<uint32_t>(i);
    }
    __device__ __forceinline__ uint32_t digit(K k) const { return static_cast<uint32_t>(k >> shift) & mask; }
    __device__ __forceinline__ void store(uint32_t dst, K k, uint32_t v) const {
        out_k[dst] = k;
        out_v[dst] = v;
    }
    __device__ __forceinline__ void placed(int64_t, uint32_t) const {}
};

template <typename K>
struct SortNextPolicy {
    using KeyT = K;
    static constexpr bool kStageDigit = false;
    const K* in_k;
    const uint32_t* in_v;
    K* out_k;
    uint32_t* out_v;
    int shift;
    uint32_t mask;
    __device__ __forceinline__ K load_key(int64_t i) const { return in_k[i]; }
    __device__ __forceinline__ void load(int64_t i, K& k, uint32_t& v) const {
        k = in_k[i];
        v = in_v[i];
    }
    __device__ __forceinline__ uint32_t digit(K k) const { return static_cast<uint32_t>(k >> shift) & mask; }
    __device__ __forceinline__ void store(uint32_t dst, K k, uint32_t v) const {
        out_k[dst] = k;
        out_v[dst] = v;
    }
    __device__ __forceinline__ void placed(int64_t, uint32_t) const {}
};

// 32-bit sort keys travel between the passes as (key, position) pairs in ONE array: a run of items that a tile appends to
// a bin is then one contiguous piece instead of one piece in each of two arrays.  The scatter passes are bound by the number
// of such pieces (every one leaves the CU, and mostly L2, as a partial line of its own), not by their bytes.  The last pass
// writes the sorted keys and the positions (the occurrence list, an output) as arrays of their own.
template <bool FIRST, bool LAST>
struct SortPairPolicy {
    using KeyT = uint32_t;
    static constexpr bool kStageDigit = false;
    const int64_t* keys;  // FIRST: the batch
    const uint2* in;      // otherwise: the previous pass's pairs
    uint2* out;           // not LAST
    uint32_t* out_k;      // LAST
    uint32_t* out_v;
    int shift;
    uint32_t mask;
    __device__ __forceinline__ uint32_t load_key(int64_t i) const {
        if (FIRST) return static_cast<uint32_t>(keys[i]);
        return in[i].x;
    }
    __device__ __forceinline__ void load(int64_t i, uint32_t& k, uint32_t& v) const {
        if (FIRST) {
            k = static_cast<uint32_t>(keys[i]);
            v = static_cast<uint32_t>(i);
        } else {
            const uint2 t = in[i];
            k = t.x;
            v = t.y;
        }
    }
    __device__ __forceinline__ uint32_t digit(uint32_t k) const { return (k >> shift) & mask; }
    __device__ __forceinline__ void store(uint32_t dst, uint32_t k, uint32_t v) const {
        if (LAST) {
            out_k[dst] = k;
            out_v[dst] = v;
        } else {
            out[dst] = make_uint2(k, v);
        }
    }
    __device__ __forceinline__ void placed(int64_t, uint32_t) const {}
};

// ---- after the sort: segment heads -> ranks ------------------------------------------------------------

#ifndef NP_HEAD_THREADS
#define NP_HEAD_THREADS 256
#endif
constexpr int kHeadThreads = NP_HEAD_THREADS;
#ifndef NP_HEAD_IPT
#define NP_HEAD_IPT 8
#endif
constexpr int kHeadIPT = NP_HEAD_IPT;
constexpr int kHeadTile = kHeadThreads * kHeadIPT;
#ifndef NP_EMIT_CHUNKS
#define NP_EMIT_CHUNKS 512  // measured: 0.82 ms with 1024 blocks, 0.79 with 384, 0.66 with 512 or 256
#endif
constexpr int kEmitChunks = NP_EMIT_CHUNKS;  // blocks of the head-count and emit kernels

// First sorted position of chunk c of the head-count / emit kernels: whole tiles of kHeadTile positions, cut into
// num_chunks runs that differ by at most one tile.
__host__ __device__ __forceinline__ int64_t head_chunk_begin(int num_tiles, int num_chunks, int c) {
    return (static_cast<int64_t>(c) * num_tiles / num_chunks) * kHeadTile;
}

// Number of segment heads (sorted[i] != sorted[i-1], position 0 is a head) in every chunk of the emit kernel.  A pure
// streaming read, so it runs with four times the emit kernel's threads per block (0.058 -> 0.041 ms).
constexpr int kCountThreads = 1024;
template <typename K>
__global__ void __launch_bounds__(kCountThreads)
dedup_count_heads_kernel(const K* __restrict__ sorted, int n, int num_tiles, int num_chunks, int* __restrict__ chunk_heads) {
    __shared__ int wsum[kCountThreads / kWave];
    const int64_t lo = head_chunk_begin(num_tiles, num_chunks, blockIdx.x);
    int64_t hi = head_chunk_begin(num_tiles, num_chunks, blockIdx.x + 1);
    if (hi > n) hi = n;
    int cnt = 0;
    for (int64_t base = lo; base < hi; base += static_cast<int64_t>(kCountThreads) * 8) {
        K cur[8], prv[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {  // sixteen independent loads in flight per thread
            const int64_t i = base + q * kCountThreads + threadIdx.x;
            cur[q] = K(0);
            prv[q] = K(0);
            if (i < hi) {
                cur[q] = sorted[i];
                if (i > 0) prv[q] = sorted[i - 1];
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int64_t i = base + q * kCountThreads + threadIdx.x;
            if (i < hi) cnt += (i == 0 || cur[q] != prv[q]) ? 1 : 0;
        }
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) cnt += __shfl_xor(cnt, d, kWave);
    if (__lane_id() == 0) wsum[threadIdx.x / kWave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
        for (int i = 0; i < kCountThreads / kWave; ++i) s += wsum[i];
        chunk_heads[blockIdx.x] = s;
    }
}

// One block per chunk: ranks every position, writes unique / occ_offsets at heads and scatters inverse.
template <typename K>
__global__ void __launch_bounds__(kHeadThreads)
dedup_emit_kernel(const K* __restrict__ sorted, const int32_t* __restrict__ occ, int n, int num_tiles, int num_chunks,
                  const int* __restrict__ chunk_heads, int64_t* __restrict__ unique, int32_t* __restrict__ inverse,
                  int32_t* __restrict__ occ_offsets, int32_t* __restrict__ d_num_unique) {
    __shared__ int scan_tmp[16];
    __shared__ int red[kHeadThreads / kWave];
    const int c = blockIdx.x;
    // heads in all earlier chunks (num_chunks <= kEmitChunks, a handful of loads per thread)
    int before = 0, all = 0;
    for (int i = threadIdx.x; i < num_chunks; i += kHeadThreads) {
        const int h = chunk_heads[i];
        all += h;
        if (i < c) before += h;
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        before += __shfl_xor(before, d, kWave);
        all += __shfl_xor(all, d, kWave);
    }
    if (__lane_id() == 0) red[threadIdx.x / kWave] = before;
    __syncthreads();
    before = 0;
    for (int i = 0; i < kHeadThreads / kWave; ++i) before += red[i];
    __syncthreads();
    if (c == 0) {
        if (__lane_id() == 0) red[threadIdx.x / kWave] = all;
        __syncthreads();
        if (threadIdx.x == 0) {
            int U = 0;
            for (int i = 0; i < kHeadThreads / kWave; ++i) U += red[i];
            *d_num_unique = U;
            occ_offsets[U] = n;
        }
    }
    const int64_t lo = head_chunk_begin(num_tiles, num_chunks, c);
    int64_t hi = head_chunk_begin(num_tiles, num_chunks, c + 1);
    if (hi > n) hi = n;
    int running = before;  // heads before the current tile
    for (int64_t tile = lo; tile < hi; tile += kHeadTile) {
        // blocked arrangement: thread t owns positions tile + t*IPT .. +IPT-1, so a thread-level scan is in order
        const int64_t p0 = tile + static_cast<int64_t>(threadIdx.x) * kHeadIPT;
        K k[kHeadIPT];
        int flag[kHeadIPT];
        K prev = K(0);
        if (p0 > 0 && p0 < hi) prev = sorted[p0 - 1];
        int local = 0;
#pragma unroll
        for (int i = 0; i < kHeadIPT; ++i) {
            const int64_t p = p0 + i;
            flag[i] = 0;
            if (p < hi) {
                k[i] = sorted[p];
                flag[i] = (p == 0 || k[i] != prev) ? 1 : 0;
                prev = k[i];
            }
            local += flag[i];
        }
        int total;
        int ex = block_excl_scan<kHeadThreads / kWave>(local, scan_tmp, &total);
        int rank = running + ex;  // heads strictly before p0
#pragma unroll
        for (int i = 0; i < kHeadIPT; ++i) {
            const int64_t p = p0 + i;
            if (p < hi) {
                rank += flag[i];
                const int u = rank - 1;
                if (flag[i]) {
                    unique[u] = static_cast<int64_t>(k[i]);
                    occ_offsets[u] = static_cast<int32_t>(p);
                }
                // a plain store: L2 merges the partial lines (a non-temporal one doubles the kernel's time)
                if (inverse) inverse[occ[p]] = u;
            }
        }
        running += total;
    }
}

// ---- the same ranking with one block per tile, tiles run in an order that lets the inverse map's scattered stores merge ----
//
// inverse[occ[p]] = rank is a scatter of n 4-byte words.  Inside the segment of one key the targets ascend, and the
// segments of all popular keys cover the same range of lookups, so tiles of different popular keys that lie at the same
// height of the batch write into the same cache lines.  Run side by side on one die they fill those lines in L2 before
// they are written back; run whenever their chunk comes up (the chunked kernel above) every store leaves L2 as a
// 32-byte sector of its own.  A tile counts as ordered when all its positions hold one key; its bucket is the band of
// the batch its first lookup lies in.  Tiles of mixed keys follow in index order.
// Measured on 42 M lookups (Zipf 1.05 over 800 M rows): the kernel 0.69 -> 0.54 ms, bytes written 1.66 -> 1.42 GB.  Only
// the few most popular keys gain: a tile of 1024 lookups of a key with a 1/2000 share is spread over two million
// lookups of the batch, more than L2 holds, so most stores still leave as single sectors (42 M x 32 bytes = 1.34 GB is
// the floor of a 4-byte scatter on this memory system).
// Built, bit-exact and slower: a hash table (key -> rank, 1 MB, resident in L2) of the keys with more than 32 lookups, which
// receive two thirds of the lookups, filled from the counts; one pass over the batch in its own order looks every key up
// and writes the ranks it finds with coalesced stores, and the scatter skips the positions that pass covers.  The scatter
// 0.54 -> 0.38 ms, but the pass takes 0.30 ms (every probe moves a 128-byte line from L2 to L1, 5.4 GB in all): np_dedup 1.90 ms
// against 1.79.  A random 4-byte read costs this memory system as much as a random 4-byte write.
constexpr int kOrdIPT = 4;
constexpr int kOrdTile = kHeadThreads * kOrdIPT;  // 1024 sorted positions
constexpr int kOrdBuckets = 1024;
// Below tune_get(kTuneEmitOrderMinN) lookups (4 M unless changed) the five extra launches cost more than the merged stores return.

// Heads per tile and the tile's bucket; one wave per tile (sixteen positions per lane), four tiles per block, no LDS.
template <typename K>
__global__ void __launch_bounds__(kHeadThreads)
dedup_tile_heads_kernel(const K* __restrict__ sorted, const int32_t* __restrict__ occ, int n, int num_tiles,
                        int32_t* __restrict__ tile_heads, uint32_t* __restrict__ tile_bucket) {
    constexpr int PER_LANE = kOrdTile / kWave;
    const int tile = blockIdx.x * (kHeadThreads / kWave) + threadIdx.x / kWave;
    if (tile >= num_tiles) return;  // whole waves leave together
    const int lane = __lane_id();
    const int64_t first = static_cast<int64_t>(tile) * kOrdTile;
    K cur[PER_LANE], prv[PER_LANE];
    // unconditional loads from clamped positions (conditional ones are issued one at a time), validity applied afterwards
#pragma unroll
    for (int q = 0; q < PER_LANE; ++q) {
        const int64_t i = first + q * kWave + lane;
        const int64_t ic = i < n ? i : n - 1;
        cur[q] = sorted[ic];
        prv[q] = sorted[ic > 0 ? ic - 1 : 0];
    }
    int cnt = 0;
#pragma unroll
    for (int q = 0; q < PER_LANE; ++q) {
        const int64_t i = first + q * kWave + lane;
        if (i < n) cnt += (i == 0 || cur[q] != prv[q]) ? 1 : 0;
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) cnt += __shfl_xor(cnt, d, kWave);
    if (lane == 0) {
        tile_heads[tile] = cnt;
        // a full tile whose positions all hold one key (no head after its first position): the band of its first lookup
        const bool full = first + kOrdTile <= n;
        const bool one_key = full && cnt <= 1 && (cnt == 0 || first == 0 || cur[0] != prv[0]);
        tile_bucket[tile] = one_key ? static_cast<uint32_t>((static_cast<uint64_t>(static_cast<uint32_t>(occ[first])) * kOrdBuckets) /
                                                            static_cast<uint32_t>(n))
                                    : static_cast<uint32_t>(kOrdBuckets);
    }
}

// Exclusive prefix sums of the per-tile head counts (one block); also the number of distinct keys and the closing offset.
__global__ void __launch_bounds__(1024)
dedup_tile_scan_kernel(const int32_t* __restrict__ tile_heads, int num_tiles, int n, int32_t* __restrict__ tile_base,
                       int32_t* __restrict__ occ_offsets, int32_t* __restrict__ d_num_unique) {
    __shared__ int scan_tmp[32];
    int running = 0;
    for (int base = 0; base < num_tiles; base += 1024 * 4) {
        int v[4], local = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {  // blocked: thread t owns tiles base + 4t .. 4t + 3
            const int i = base + static_cast<int>(threadIdx.x) * 4 + q;
            v[q] = i < num_tiles ? tile_heads[i] : 0;
            local += v[q];
        }
        int total;
        int ex = running + block_excl_scan<1024 / kWave>(local, scan_tmp, &total);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = base + static_cast<int>(threadIdx.x) * 4 + q;
            if (i < num_tiles) tile_base[i] = ex;
            ex += v[q];
        }
        running += total;
    }
    if (threadIdx.x == 0) {
        *d_num_unique = running;
        occ_offsets[running] = n;
    }
}

// Partition policy over the precomputed buckets; the payload is the tile index.
struct EmitOrderPolicy {
    using KeyT = uint32_t;
    static constexpr bool kStageDigit = false;
    const uint32_t* tile_bucket;
    int32_t* order;
    __device__ __forceinline__ uint32_t load_key(int64_t i) const { return tile_bucket[i]; }
    __device__ __forceinline__ void load(int64_t i, uint32_t& k, uint32_t& v) const {
        k = tile_bucket[i];
        v = static_cast<uint32_t>(i);
    }
    __device__ __forceinline__ uint32_t digit(uint32_t k) const { return k; }
    __device__ __forceinline__ void store(uint32_t dst, uint32_t, uint32_t v) const { order[dst] = static_cast<int32_t>(v); }
    __device__ __forceinline__ void placed(int64_t, uint32_t) const {}
};

// One block per tile, in the given order: die x (blocks x, x + 8, ...) first runs its contiguous share of the ordered
// tiles, i.e. one eighth of the bands of the batch, then every eighth of the others.
template <typename K>
__global__ void __launch_bounds__(kHeadThreads)
dedup_emit_tiles_kernel(const K* __restrict__ sorted, const int32_t* __restrict__ occ, int n, int num_tiles,
                        const int32_t* __restrict__ tile_base, const int32_t* __restrict__ order,
                        const int32_t* __restrict__ order_offsets, int64_t* __restrict__ unique, int32_t* __restrict__ inverse,
                        int32_t* __restrict__ occ_offsets) {
    __shared__ int scan_tmp[16];
    // (a fixed number of blocks walking the tiles instead of one block per tile is slower: 0.57-0.59 against 0.54 ms)
    int tile;
    {
        const int nh = order_offsets[kOrdBuckets];
        const int nc = num_tiles - nh;
        const int hc = (nh + kNumXcd - 1) / kNumXcd;
        const int x = blockIdx.x % kNumXcd, sl = blockIdx.x / kNumXcd;
        int k;
        if (sl < hc) {
            k = x * hc + sl;
            if (k >= nh) return;
        } else {
            const int kc = (sl - hc) * kNumXcd + x;
            if (kc >= nc) return;
            k = nh + kc;
        }
        tile = order[k];
    }
    // blocked arrangement: thread t owns positions p0 .. p0 + kOrdIPT - 1
    const int64_t p0 = static_cast<int64_t>(tile) * kOrdTile + static_cast<int64_t>(threadIdx.x) * kOrdIPT;
    K k[kOrdIPT];
    int flag[kOrdIPT], j[kOrdIPT];
    K prev = K(0);
    if (p0 > 0 && p0 < n) prev = sorted[p0 - 1];
    int local = 0;
    // (conditional loads on purpose: issued back to back from clamped positions this kernel is slower, 0.66 against 0.53 ms
    // on 42 M lookups; its time is in the scattered stores, and those do better when the waves do not all issue them at once)
#pragma unroll
    for (int i = 0; i < kOrdIPT; ++i) {
        const int64_t p = p0 + i;
        flag[i] = 0;
        j[i] = 0;
        k[i] = K(0);
        if (p < n) {
            k[i] = sorted[p];
            j[i] = occ[p];
        }
    }
#pragma unroll
    for (int i = 0; i < kOrdIPT; ++i) {
        const int64_t p = p0 + i;
        if (p < n) {
            flag[i] = (p == 0 || k[i] != prev) ? 1 : 0;
            prev = k[i];
        }
        local += flag[i];
    }
    int total;
    int rank = tile_base[tile] + block_excl_scan<kHeadThreads / kWave>(local, scan_tmp, &total);  // heads strictly before p0
#pragma unroll
    for (int i = 0; i < kOrdIPT; ++i) {
        const int64_t p = p0 + i;
        if (p < n) {
            rank += flag[i];
            const int u = rank - 1;
            if (flag[i]) {
                unique[u] = static_cast<int64_t>(k[i]);
                occ_offsets[u] = static_cast<int32_t>(p);
            }
            inverse[j[i]] = u;  // a plain store: the lines are completed in L2
        }
    }
}

__global__ void __launch_bounds__(256)
dedup_counts_kernel(const int32_t* __restrict__ occ_offsets, const int32_t* __restrict__ d_num_unique, int n, int32_t* __restrict__ counts) {
    const int U = device_count(d_num_unique, n);
    for (int u = blockIdx.x * blockDim.x + threadIdx.x; u < U; u += gridDim.x * blockDim.x)
        counts[u] = occ_offsets[u + 1] - occ_offsets[u];
}

__global__ void dedup_empty_kernel(int32_t* occ_offsets, int32_t* d_num_unique) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *d_num_unique = 0;
        occ_offsets[0] = 0;
    }
}

struct DedupWs {
    size_t key_bytes;   // one key buffer
    size_t total;
    ChunkPlan plan;
    PassPlan passes;
    int max_bins;
};

inline DedupWs dedup_ws_layout(int32_t n, int32_t key_bits) {
    DedupWs w;
    w.plan = make_chunk_plan(n);
    w.passes = make_pass_plan(key_bits);
    w.max_bins = 1 << w.passes.bits[0];
    // 32-bit sort keys: two buffers of (key, position) pairs; 64-bit: two key buffers and a second position buffer
    w.key_bytes = align_up(8 * static_cast<size_t>(n), 256);
    w.total = 2 * w.key_bytes + (key_bits <= 32 ? 0 : align_up(4 * static_cast<size_t>(n), 256))
              + align_up(4 * part_hist_elems(w.plan, w.max_bins), 256)        // histogram matrix
              + align_up(4 * static_cast<size_t>(w.max_bins), 256)            // bin totals
              + align_up(4 * static_cast<size_t>(kEmitChunks), 256);          // heads per chunk
    // the tile-ordered emit: heads, bases and order of the tiles, bucket offsets, its own partition scratch
    const size_t ord_tiles = (static_cast<size_t>(n) + kOrdTile - 1) / kOrdTile;
    w.total += 4 * align_up(4 * ord_tiles, 256) + align_up(4 * static_cast<size_t>(kOrdBuckets + 2), 256)
               + align_up(4 * part_hist_elems(make_chunk_plan(static_cast<int64_t>(ord_tiles)), kOrdBuckets + 1), 256)
               + align_up(4 * static_cast<size_t>(kOrdBuckets + 1), 256);
    return w;
}

template <typename K>
int dedup_impl(const int64_t* keys, int32_t n, int32_t key_bits, int64_t* unique, int32_t* inverse, int32_t* counts,
               int32_t* occ_offsets, int32_t* occ, int32_t* d_num_unique, void* ws, hipStream_t stream) {
    const DedupWs L = dedup_ws_layout(n, key_bits);
    WsCursor cur(ws);
    unsigned char* buf[2] = {cur.take<unsigned char>(L.key_bytes), cur.take<unsigned char>(L.key_bytes)};
    uint32_t* vtmp = sizeof(K) == 4 ? nullptr : cur.take<uint32_t>(n);
    uint32_t* H = cur.take<uint32_t>(part_hist_elems(L.plan, L.max_bins));
    uint32_t* bin_total = cur.take<uint32_t>(L.max_bins);
    int* chunk_heads = cur.take<int>(kEmitChunks);
    uint32_t* vocc = reinterpret_cast<uint32_t*>(occ);

    const int P = L.passes.passes;
    const K* sorted;
    if constexpr (sizeof(K) == 4) {
        // pass p writes pairs into buf[p % 2]; the last pass reads buf[(P - 2) % 2] and puts the sorted keys into the other one
        uint2* pairs[2] = {reinterpret_cast<uint2*>(buf[0]), reinterpret_cast<uint2*>(buf[1])};
        uint32_t* sorted_out = reinterpret_cast<uint32_t*>(buf[(P - 1) % 2]);
        for (int p = 0; p < P; ++p) {
            const int bits = L.passes.bits[p], bins = 1 << bits, shift = L.passes.shift[p];
            const uint32_t mask = static_cast<uint32_t>(bins - 1);
            const uint2* in = p > 0 ? pairs[(p - 1) % 2] : nullptr;
            const bool first = p == 0, last = p == P - 1;
#define NP_SORT_PASS(F, Z)                                                                                                   \
    do {                                                                                                                     \
        SortPairPolicy<F, Z> pol{keys, in, pairs[p % 2], sorted_out, vocc, shift, mask};                                      \
        run_partition_pass(pol, n, nullptr, bins, bits, L.plan, H, bin_total, nullptr, nullptr, stream, "dedup_sort_hist",   \
                           "dedup_sort_colscan", "dedup_sort_scatter");                                                      \
    } while (0)
            if (first && last) NP_SORT_PASS(true, true);
            else if (first) NP_SORT_PASS(true, false);
            else if (last) NP_SORT_PASS(false, true);
            else NP_SORT_PASS(false, false);
#undef NP_SORT_PASS
        }
        sorted = sorted_out;
    } else {
        K* kbuf[2] = {reinterpret_cast<K*>(buf[0]), reinterpret_cast<K*>(buf[1])};
        // payload buffers alternate so that the last pass lands in occ
        for (int p = 0; p < P; ++p) {
            const int bits = L.passes.bits[p], bins = 1 << bits;
            const uint32_t mask = static_cast<uint32_t>(bins - 1);
            uint32_t* vout = ((P - 1 - p) % 2 == 0) ? vocc : vtmp;
            K* kout = kbuf[p % 2];
            if (p == 0) {
                SortFirstPolicy<K> pol{keys, kout, vout, L.passes.shift[p], mask};
                run_partition_pass(pol, n, nullptr, bins, bits, L.plan, H, bin_total, nullptr, nullptr, stream,
                                   "dedup_sort_hist", "dedup_sort_colscan", "dedup_sort_scatter");
            } else {
                const uint32_t* vin = ((P - p) % 2 == 0) ? vocc : vtmp;
                SortNextPolicy<K> pol{kbuf[(p - 1) % 2], vin, kout, vout, L.passes.shift[p], mask};
                run_partition_pass(pol, n, nullptr, bins, bits, L.plan, H, bin_total, nullptr, nullptr, stream,
                                   "dedup_sort_hist", "dedup_sort_colscan", "dedup_sort_scatter");
            }
        }
        sorted = kbuf[(P - 1) % 2];
    }
    if (inverse && n >= tune_get(kTuneEmitOrderMinN)) {
        const int ord_tiles = static_cast<int>((static_cast<int64_t>(n) + kOrdTile - 1) / kOrdTile);
        int32_t* tile_heads = cur.take<int32_t>(ord_tiles);
        int32_t* tile_base = cur.take<int32_t>(ord_tiles);
        int32_t* order = cur.take<int32_t>(ord_tiles);
        uint32_t* tile_bucket = cur.take<uint32_t>(ord_tiles);
        int32_t* order_offsets = cur.take<int32_t>(kOrdBuckets + 2);
        const ChunkPlan oplan = make_chunk_plan(ord_tiles);
        uint32_t* oH = cur.take<uint32_t>(part_hist_elems(oplan, kOrdBuckets + 1));
        uint32_t* obin = cur.take<uint32_t>(kOrdBuckets + 1);
        constexpr int kTilesPerBlock = kHeadThreads / kWave;
        NP_LAUNCH("dedup_tile_heads", dedup_tile_heads_kernel<K>, dim3((ord_tiles + kTilesPerBlock - 1) / kTilesPerBlock),
                  dim3(kHeadThreads), 0, stream, sorted, occ, n, ord_tiles, tile_heads, tile_bucket);
        NP_LAUNCH("dedup_tile_scan", dedup_tile_scan_kernel, dim3(1), dim3(1024), 0, stream, tile_heads, ord_tiles, n, tile_base,
                  occ_offsets, d_num_unique);
        EmitOrderPolicy pol{tile_bucket, order};
        run_partition_pass(pol, ord_tiles, nullptr, kOrdBuckets + 1, 11, oplan, oH, obin, nullptr, order_offsets, stream,
                           "dedup_order_hist", "dedup_order_colscan", "dedup_order_scatter");
        const unsigned grid = static_cast<unsigned>((ord_tiles + 2 * kNumXcd + kNumXcd - 1) / kNumXcd * kNumXcd);
        NP_LAUNCH("dedup_emit", dedup_emit_tiles_kernel<K>, dim3(grid), dim3(kHeadThreads), 0, stream, sorted, occ, n, ord_tiles,
                  tile_base, order, order_offsets, unique, inverse, occ_offsets);
    } else {
        // chunks of whole head-tiles, at most kEmitChunks of them
        const int num_tiles = static_cast<int>((static_cast<int64_t>(n) + kHeadTile - 1) / kHeadTile);
        const int num_chunks = num_tiles < kEmitChunks ? num_tiles : kEmitChunks;
        NP_LAUNCH("dedup_count_heads", dedup_count_heads_kernel<K>, dim3(num_chunks), dim3(kCountThreads), 0, stream, sorted, n,
                  num_tiles, num_chunks, chunk_heads);
        NP_LAUNCH("dedup_emit", dedup_emit_kernel<K>, dim3(num_chunks), dim3(kHeadThreads), 0, stream, sorted, occ, n,
                  num_tiles, num_chunks, chunk_heads, unique, inverse, occ_offsets, d_num_unique);
    }
    int cgrid = (n + 255) / 256;
    if (cgrid > 4096) cgrid = 4096;
    NP_LAUNCH("dedup_counts", dedup_counts_kernel, dim3(cgrid), dim3(256), 0, stream, occ_offsets, d_num_unique, n, counts);
    return launch_status();
}

}  // namespace np

extern "C" {

size_t np_dedup_workspace_bytes(int32_t n, int32_t key_bits) {
    if (n <= 0 || key_bits < 1 || key_bits > 63) return 0;
    return np::dedup_ws_layout(n, key_bits).total;
}

int np_dedup(const int64_t* keys, int32_t n, int32_t key_bits, int64_t* unique, int32_t* inverse, int32_t* counts,
             int32_t* occ_offsets, int32_t* occ, int32_t* d_num_unique, void* ws, size_t ws_bytes, void* stream) {
    if (n < 0 || key_bits < 1 || key_bits > 63 || !occ_offsets || !d_num_unique) return NP_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n == 0) {
        NP_LAUNCH("dedup_empty", np::dedup_empty_kernel, dim3(1), dim3(64), 0, s, occ_offsets, d_num_unique);
        return np::launch_status();
    }
    if (!keys || !unique || !counts || !occ) return NP_ERR_INVALID_ARG;  // inverse is optional
    if (n > INT32_MAX - (1 << 20)) return NP_ERR_UNSUPPORTED;  // tile-rounded indices must stay below 2^31
    if (!np::aligned(keys, 8) || !np::aligned(unique, 8) || !np::aligned(inverse, 4) || !np::aligned(counts, 4) ||
        !np::aligned(occ_offsets, 4) || !np::aligned(occ, 4))
        return NP_ERR_INVALID_ARG;
    if (!ws || !np::aligned(ws, 256) || ws_bytes < np_dedup_workspace_bytes(n, key_bits)) return NP_ERR_WORKSPACE;
    if (key_bits <= 32)
        return np::dedup_impl<uint32_t>(keys, n, key_bits, unique, inverse, counts, occ_offsets, occ, d_num_unique, ws, s);
    return np::dedup_impl<uint64_t>(keys, n, key_bits, unique, inverse, counts, occ_offsets, occ, d_num_unique, ws, s);
}

}  // extern "C"
