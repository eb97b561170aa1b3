// Dual-buffer synchronisation (Section IV-B): before batch B_t starts its forward pass, the intersection of
// the compact key sets of B_{t-1} and B_t is computed on the keys alone, and the vectors of the common keys are
// copied from the active buffer (which holds B_{t-1}'s updates) into the prefetch buffer (filled for B_t before
// those updates).  Afterwards the prefetch buffer holds exactly the parameters a sequential run would read
// (Proposition 1, Eq. (2)).
//
//   intersect_probe  every key of B is looked up in A by binary search, tile by tile inside the slice of A that can
//                    hold the tile's keys (both lists ascend), staged in LDS; hits per chunk
//   intersect_emit   ranks the hits (block scan over a blocked arrangement) and writes the index pairs in
//                    ascending key order; deterministic, no atomics
//   sync_rows        one LPR-lane group per pair copies a row with 16-byte lane accesses
#include "np_common.hpp"

namespace np {

constexpr int kIsThreads = 256;
constexpr int kIsIPT = 8;
constexpr int kIsTile = kIsThreads * kIsIPT;
constexpr int kIsMaxChunks = 1024;

struct IsPlan {
    int num_chunks;
    int chunk_items;
};

inline IsPlan make_is_plan(int cap) {
    int64_t tiles = (static_cast<int64_t>(cap) + kIsTile - 1) / kIsTile;
    if (tiles < 1) tiles = 1;
    const int64_t tpc = (tiles + kIsMaxChunks - 1) / kIsMaxChunks;
    IsPlan p;
    p.num_chunks = static_cast<int>((tiles + tpc - 1) / tpc);
    p.chunk_items = static_cast<int>(tpc * kIsTile);
    return p;
}

constexpr int kIsStage = 4096;      // keys of A staged in LDS per tile of B (32 KB)
constexpr int kIsTileBatch = 64;    // tiles whose ranges in A are located together

// First index in [l, h) of an ascending list whose key is not below `key` (h if there is none).
__device__ __forceinline__ int lower_bound_keys(const int64_t* __restrict__ keys, int l, int h, int64_t key) {
    while (l < h) {
        const int m = l + (h - l) / 2;
        if (keys[m] < key) l = m + 1;
        else h = m;
    }
    return l;
}

// One block per chunk of B.  Both lists ascend, so a tile of kIsTile consecutive keys of B can only match inside
// [first A >= the tile's first key, first A >= the next tile's first key): that slice of A is staged in LDS
// (coalesced) and every key of the tile is located in it by binary search; a slice that does not fit is searched
// in place.  The slice boundaries of up to kIsTileBatch tiles are found together, one thread each.
__global__ void __launch_bounds__(kIsThreads)
intersect_probe_kernel(const int64_t* __restrict__ keys_a, const int32_t* __restrict__ d_num_a, const int64_t* __restrict__ keys_b,
                       const int32_t* __restrict__ d_num_b, int cap_a, int cap_b, int chunk_items, int32_t* __restrict__ found,
                       int32_t* __restrict__ chunk_hits) {
    __shared__ int64_t sa[kIsStage];
    __shared__ int bound[kIsTileBatch + 1];
    __shared__ int wsum[kIsThreads / kWave];
    const int na = device_count(d_num_a, cap_a), nb = device_count(d_num_b, cap_b);
    const int64_t lo = static_cast<int64_t>(blockIdx.x) * chunk_items;
    int64_t hi = lo + chunk_items;
    if (hi > nb) hi = nb;
    int hits = 0;
    for (int64_t batch = lo; batch < hi; batch += static_cast<int64_t>(kIsTileBatch) * kIsTile) {
        __syncthreads();  // bound[] and sa[] of the previous batch are no longer read
        if (threadIdx.x <= kIsTileBatch) {
            const int64_t first = batch + static_cast<int64_t>(threadIdx.x) * kIsTile;  // first key of tile threadIdx.x of the batch
            bound[threadIdx.x] = first < nb ? lower_bound_keys(keys_a, 0, na, keys_b[first]) : na;
        }
        __syncthreads();
        for (int t = 0; t < kIsTileBatch; ++t) {
            const int64_t tile = batch + static_cast<int64_t>(t) * kIsTile;
            if (tile >= hi) break;  // uniform
            const int a_lo = bound[t], a_hi = bound[t + 1];
            const int len = a_hi - a_lo;
            const bool staged = len <= kIsStage;
            if (staged)
                for (int k = threadIdx.x; k < len; k += kIsThreads) sa[k] = keys_a[a_lo + k];
            __syncthreads();
#pragma unroll
            for (int q = 0; q < kIsIPT; ++q) {
                const int64_t i = tile + q * kIsThreads + threadIdx.x;
                if (i < hi) {
                    const int64_t key = keys_b[i];
                    int f = -1;
                    if (staged) {
                        int l = 0, h = len;
                        while (l < h) {
                            const int m = (l + h) >> 1;
                            if (sa[m] < key) l = m + 1;
                            else h = m;
                        }
                        if (l < len && sa[l] == key) f = a_lo + l;
                    } else {
                        const int l = lower_bound_keys(keys_a, a_lo, a_hi, key);
                        if (l < a_hi && keys_a[l] == key) f = l;
                    }
                    found[i] = f;
                    hits += f >= 0 ? 1 : 0;
                }
            }
            __syncthreads();  // sa[] is rewritten by the next tile
        }
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) hits += __shfl_xor(hits, d, kWave);
    if (__lane_id() == 0) wsum[threadIdx.x / kWave] = hits;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
        for (int i = 0; i < kIsThreads / kWave; ++i) s += wsum[i];
        chunk_hits[blockIdx.x] = s;
    }
}

__global__ void __launch_bounds__(kIsThreads)
intersect_emit_kernel(const int32_t* __restrict__ d_num_b, int cap_b, int chunk_items, int num_chunks, const int32_t* __restrict__ found,
                      const int32_t* __restrict__ chunk_hits, int32_t* __restrict__ idx_a, int32_t* __restrict__ idx_b,
                      int32_t* __restrict__ d_num_common) {
    __shared__ int scan_tmp[16];
    __shared__ int red[2][kIsThreads / kWave];
    const int c = blockIdx.x;
    const int nb = device_count(d_num_b, cap_b);
    int before = 0, all = 0;
    for (int i = threadIdx.x; i < num_chunks; i += kIsThreads) {
        const int h = chunk_hits[i];
        all += h;
        if (i < c) before += h;
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        before += __shfl_xor(before, d, kWave);
        all += __shfl_xor(all, d, kWave);
    }
    if (__lane_id() == 0) {
        red[0][threadIdx.x / kWave] = before;
        red[1][threadIdx.x / kWave] = all;
    }
    __syncthreads();
    before = 0;
    all = 0;
    for (int i = 0; i < kIsThreads / kWave; ++i) {
        before += red[0][i];
        all += red[1][i];
    }
    if (c == 0 && threadIdx.x == 0) *d_num_common = all;
    const int64_t lo = static_cast<int64_t>(c) * chunk_items;
    int64_t hi = lo + chunk_items;
    if (hi > nb) hi = nb;
    int running = before;
    for (int64_t tile = lo; tile < hi; tile += kIsTile) {
        const int64_t p0 = tile + static_cast<int64_t>(threadIdx.x) * kIsIPT;  // blocked: a thread's items are consecutive
        int f[kIsIPT];
        int local = 0;
#pragma unroll
        for (int i = 0; i < kIsIPT; ++i) {
            f[i] = p0 + i < hi ? found[p0 + i] : -1;
            local += f[i] >= 0 ? 1 : 0;
        }
        int total;
        int rank = running + block_excl_scan<kIsThreads / kWave>(local, scan_tmp, &total);
#pragma unroll
        for (int i = 0; i < kIsIPT; ++i) {
            if (f[i] >= 0) {
                idx_a[rank] = f[i];
                idx_b[rank] = static_cast<int32_t>(p0 + i);
                ++rank;
            }
        }
        running += total;
    }
}

template <int LPR, int NV>
__global__ void __launch_bounds__(256)
sync_rows_kernel(const float* __restrict__ src, const int32_t* __restrict__ src_idx, float* __restrict__ dst,
                 const int32_t* __restrict__ dst_idx, const int32_t* __restrict__ d_count, int cap, int dim) {
    constexpr int GPB = 256 / LPR;
    const int r = threadIdx.x % LPR;
    const int words = dim / 4;
    const int count = device_count(d_count, cap);
    for (int64_t p = static_cast<int64_t>(blockIdx.x) * GPB + threadIdx.x / LPR; p < count; p += static_cast<int64_t>(gridDim.x) * GPB) {
        const float4* s = reinterpret_cast<const float4*>(src + static_cast<size_t>(src_idx[p]) * dim);
        float4* d = reinterpret_cast<float4*>(dst + static_cast<size_t>(dst_idx[p]) * dim);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int wv = r + v * LPR;
            if (wv < words) d[wv] = s[wv];
        }
    }
}

template <int LPR, int NV>
void sync_rows_launch(const float* src, const int32_t* src_idx, float* dst, const int32_t* dst_idx, const int32_t* d_count,
                      int cap, int dim, hipStream_t stream) {
    constexpr int GPB = 256 / LPR;
    int64_t want = (static_cast<int64_t>(cap) + GPB - 1) / GPB;
    const unsigned grid = static_cast<unsigned>(want < 32768 ? want : 32768);
    NP_LAUNCH("sync_rows", (sync_rows_kernel<LPR, NV>), dim3(grid), dim3(256), 0, stream, src, src_idx, dst, dst_idx, d_count, cap, dim);
}

}  // namespace np

extern "C" {

size_t np_intersect_workspace_bytes(int32_t cap_b) {
    if (cap_b <= 0) return 256;
    return np::align_up(4 * static_cast<size_t>(cap_b), 256) + np::align_up(4 * static_cast<size_t>(np::kIsMaxChunks), 256);
}

int np_intersect(const int64_t* keys_a, const int32_t* d_num_a, int32_t cap_a, const int64_t* keys_b,
                 const int32_t* d_num_b, int32_t cap_b, int32_t* idx_a, int32_t* idx_b, int32_t* d_num_common, void* ws,
                 size_t ws_bytes, void* stream) {
    if (cap_a < 0 || cap_b < 0 || !d_num_a || !d_num_b || !d_num_common) return NP_ERR_INVALID_ARG;
    if ((cap_a > 0 && !keys_a) || (cap_b > 0 && (!keys_b || !idx_a || !idx_b))) return NP_ERR_INVALID_ARG;
    if (!np::aligned(keys_a, 8) || !np::aligned(keys_b, 8)) return NP_ERR_INVALID_ARG;
    if (!ws || !np::aligned(ws, 256) || ws_bytes < np_intersect_workspace_bytes(cap_b)) return NP_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const np::IsPlan plan = np::make_is_plan(cap_b);
    np::WsCursor cur(ws);
    int32_t* found = cur.take<int32_t>(cap_b > 0 ? cap_b : 1);
    int32_t* chunk_hits = cur.take<int32_t>(np::kIsMaxChunks);
    NP_LAUNCH("intersect_probe", np::intersect_probe_kernel, dim3(plan.num_chunks), dim3(np::kIsThreads), 0, s, keys_a, d_num_a, keys_b,
              d_num_b, cap_a, cap_b, plan.chunk_items, found, chunk_hits);
    NP_LAUNCH("intersect_emit", np::intersect_emit_kernel, dim3(plan.num_chunks), dim3(np::kIsThreads), 0, s, d_num_b, cap_b, plan.chunk_items,
              plan.num_chunks, found, chunk_hits, idx_a, idx_b, d_num_common);
    return np::launch_status();
}

int np_sync_rows(const float* src_rows, const int32_t* src_idx, float* dst_rows, const int32_t* dst_idx,
                 const int32_t* d_count, int32_t cap, int32_t dim, void* stream) {
    if (cap < 0 || !d_count) return NP_ERR_INVALID_ARG;
    if (dim < 4 || dim % 4 != 0 || dim > NP_MAX_DIM) return NP_ERR_UNSUPPORTED;
    if (cap == 0) return NP_OK;
    if (!src_rows || !src_idx || !dst_rows || !dst_idx || !np::aligned(src_rows, 16) || !np::aligned(dst_rows, 16))
        return NP_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int words = dim / 4;
    if (words <= 4) np::sync_rows_launch<4, 1>(src_rows, src_idx, dst_rows, dst_idx, d_count, cap, dim, s);
    else if (words <= 8) np::sync_rows_launch<8, 1>(src_rows, src_idx, dst_rows, dst_idx, d_count, cap, dim, s);
    else if (words <= 16) np::sync_rows_launch<16, 1>(src_rows, src_idx, dst_rows, dst_idx, d_count, cap, dim, s);
    else if (words <= 32) np::sync_rows_launch<32, 1>(src_rows, src_idx, dst_rows, dst_idx, d_count, cap, dim, s);
    else if (words <= 64) np::sync_rows_launch<64, 1>(src_rows, src_idx, dst_rows, dst_idx, d_count, cap, dim, s);
    else if (words <= 128) np::sync_rows_launch<64, 2>(src_rows, src_idx, dst_rows, dst_idx, d_count, cap, dim, s);
    else np::sync_rows_launch<64, 4>(src_rows, src_idx, dst_rows, dst_idx, d_count, cap, dim, s);
    return np::launch_status();
}

}  // extern "C"
