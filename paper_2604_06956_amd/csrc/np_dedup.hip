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
    const size_t ksz = key_bits <= 32 ? 4 : 8;
    w.key_bytes = align_up(ksz * static_cast<size_t>(n), 256);
    w.total = 2 * w.key_bytes                                                 // key ping-pong
              + align_up(4 * static_cast<size_t>(n), 256)                     // second position buffer
              + align_up(4 * part_hist_elems(w.plan, w.max_bins), 256)        // histogram matrix
              + align_up(4 * static_cast<size_t>(w.max_bins), 256)            // bin totals
              + align_up(4 * static_cast<size_t>(kEmitChunks), 256);          // heads per chunk
    return w;
}

template <typename K>
int dedup_impl(const int64_t* keys, int32_t n, int32_t key_bits, int64_t* unique, int32_t* inverse, int32_t* counts,
               int32_t* occ_offsets, int32_t* occ, int32_t* d_num_unique, void* ws, hipStream_t stream) {
    const DedupWs L = dedup_ws_layout(n, key_bits);
    WsCursor cur(ws);
    K* kbuf[2] = {cur.take<K>(L.key_bytes / sizeof(K)), cur.take<K>(L.key_bytes / sizeof(K))};
    uint32_t* vtmp = cur.take<uint32_t>(n);
    uint32_t* H = cur.take<uint32_t>(part_hist_elems(L.plan, L.max_bins));
    uint32_t* bin_total = cur.take<uint32_t>(L.max_bins);
    int* chunk_heads = cur.take<int>(kEmitChunks);
    uint32_t* vocc = reinterpret_cast<uint32_t*>(occ);

    // payload buffers alternate so that the last pass lands in occ
    const int P = L.passes.passes;
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
    const K* sorted = kbuf[(P - 1) % 2];
    // chunks of whole head-tiles, at most kEmitChunks of them
    const int num_tiles = static_cast<int>((static_cast<int64_t>(n) + kHeadTile - 1) / kHeadTile);
    const int num_chunks = num_tiles < kEmitChunks ? num_tiles : kEmitChunks;
    NP_LAUNCH("dedup_count_heads", dedup_count_heads_kernel<K>, dim3(num_chunks), dim3(kCountThreads), 0, stream, sorted, n,
              num_tiles, num_chunks, chunk_heads);
    NP_LAUNCH("dedup_emit", dedup_emit_kernel<K>, dim3(num_chunks), dim3(kHeadThreads), 0, stream, sorted, occ, n,
              num_tiles, num_chunks, chunk_heads, unique, inverse, occ_offsets, d_num_unique);
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
