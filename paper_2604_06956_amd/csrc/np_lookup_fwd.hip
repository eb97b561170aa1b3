// np_lookup_fwd: gather rows of the key list from the HBM-resident table and pool them per bag, or lay
// them out as a padded sequence (Section IV-A, "Embedding Retrieval" and the start of "Fwd/Bwd").
//
// A row of dim floats is dim/4 float4 words.  LPR lanes (a power of two, 4..64) share a row, each holding
// NV words, so every row access is a run of 16-byte loads from consecutive lanes.  One LPR-lane group owns
// one bag (pooled modes) or one output position (sequence mode); a 64-lane wave therefore works on
// 64/LPR bags at once.  The group first fetches the slot and key of up to LPR lookups with one lane each,
// then walks them in ascending order broadcasting the key, several row loads in flight at a time.
#include "np_common.hpp"

namespace np {

template <int LPR>
__device__ __forceinline__ int64_t group_bcast64(int64_t v, int src_in_group) {
    const int src = (__lane_id() & ~(LPR - 1)) + src_in_group;
    const int lo = __shfl(static_cast<int>(v & 0xFFFFFFFFll), src, kWave);
    const int hi = __shfl(static_cast<int>(v >> 32), src, kWave);
    return (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
}

__device__ __forceinline__ void store_words(float* p, const float4& a) { store_word_stream(p, 0, a); }

__device__ __forceinline__ void store_words(uint16_t* p, const float4& a) { store_word_stream(p, 0, a); }

constexpr int kFwdUnroll = 4;

// Table row read by lookup j: list_keys[idx[j]]; without idx the list has one entry per lookup; without list_keys the
// slot itself is the row (pooling straight from a buffer of received rows).
__device__ __forceinline__ int64_t lookup_row(const int64_t* __restrict__ list_keys, const int32_t* __restrict__ idx, int j) {
    const int64_t slot = idx ? static_cast<int64_t>(load_stream(idx + j)) : static_cast<int64_t>(j);
    return list_keys ? list_keys[slot] : slot;
}

template <int LPR, int NV, bool MEAN, typename OutT, typename TabT>
__global__ void __launch_bounds__(256)
fwd_pool_kernel(const TabT* __restrict__ table, int dim, const int64_t* __restrict__ list_keys, const int32_t* __restrict__ idx,
                const int32_t* __restrict__ bag_offsets, int num_bags, OutT* __restrict__ out) {
    constexpr int GPB = 256 / LPR;
    const int r = threadIdx.x % LPR;
    const int64_t b = static_cast<int64_t>(blockIdx.x) * GPB + threadIdx.x / LPR;
    if (b >= num_bags) return;  // whole groups leave together
    const int lo = bag_offsets[b], hi = bag_offsets[b + 1];
    const int words = dim / 4;
    float4 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);

    const int gl = __lane_id() & ~(LPR - 1);  // first lane of this group
    for (int base = lo; base < hi; base += LPR) {
        const int j = base + r;
        // one lane per lookup: slot, key and the byte offset of the row (the 64-bit multiply happens here, once
        // per lookup, instead of in every lane of the walk below)
        int64_t row_off = 0;
        if (j < hi) row_off = lookup_row(list_keys, idx, j) * static_cast<int64_t>(dim) * static_cast<int64_t>(sizeof(TabT));
        const int off_lo = static_cast<int>(row_off & 0xFFFFFFFFll), off_hi = static_cast<int>(row_off >> 32);
        const int cnt = hi - base < LPR ? hi - base : LPR;
        for (int k0 = 0; k0 < cnt; k0 += kFwdUnroll) {
            float4 x[kFwdUnroll][NV];
#pragma unroll
            for (int q = 0; q < kFwdUnroll; ++q) {
                const bool on = k0 + q < cnt;  // uniform inside the group; k0 + q < LPR always
                const uint32_t lo32 = static_cast<uint32_t>(__shfl(off_lo, gl + k0 + q, kWave));
                const uint32_t hi32 = static_cast<uint32_t>(__shfl(off_hi, gl + k0 + q, kWave));
                const TabT* src = reinterpret_cast<const TabT*>(reinterpret_cast<const char*>(table) +
                                                                ((static_cast<uint64_t>(hi32) << 32) | lo32));
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int wv = r + v * LPR;
                    x[q][v] = (on && wv < words) ? load_word(src, wv) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
#pragma unroll
            for (int q = 0; q < kFwdUnroll; ++q) {
#pragma unroll
                for (int v = 0; v < NV; ++v) {  // rows that were not loaded are zeros
                    acc[v].x += x[q][v].x;
                    acc[v].y += x[q][v].y;
                    acc[v].z += x[q][v].z;
                    acc[v].w += x[q][v].w;
                }
            }
        }
    }
    float scale = 1.f;
    if (MEAN && hi > lo) scale = 1.f / static_cast<float>(hi - lo);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int wv = r + v * LPR;
        if (wv < words) {
            float4 a = acc[v];
            if (MEAN) {
                a.x *= scale;
                a.y *= scale;
                a.z *= scale;
                a.w *= scale;
            }
            store_words(out + static_cast<size_t>(b) * dim + wv * 4, a);
        }
    }
}

// Pooling over a 16-bit (bf16 or fp16) table whose rows are a multiple of 8 elements wide: a lane owns 8 consecutive elements (one
// 16-byte load per row, as wide as an fp32 lane's), L8 lanes share a row, so a wave keeps twice as many rows in
// flight as with 8-byte lanes.  Same walk and same order of additions as fwd_pool_kernel.
__device__ __forceinline__ void widen8(const __half*, const uint4& u, float4& a, float4& b) {
    const __half2* h = reinterpret_cast<const __half2*>(&u);
    a = make_float4(__low2float(h[0]), __high2float(h[0]), __low2float(h[1]), __high2float(h[1]));
    b = make_float4(__low2float(h[2]), __high2float(h[2]), __low2float(h[3]), __high2float(h[3]));
}

__device__ __forceinline__ void widen8(const uint16_t*, const uint4& u, float4& a, float4& b) {
    a = make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                    __uint_as_float(u.y & 0xFFFF0000u));
    b = make_float4(__uint_as_float(u.z << 16), __uint_as_float(u.z & 0xFFFF0000u), __uint_as_float(u.w << 16),
                    __uint_as_float(u.w & 0xFFFF0000u));
}

template <int L8, int NV8, bool MEAN, typename OutT, typename TabT>
__global__ void __launch_bounds__(256)
fwd_pool_x8_kernel(const TabT* __restrict__ table, int dim, const int64_t* __restrict__ list_keys,
                       const int32_t* __restrict__ idx, const int32_t* __restrict__ bag_offsets, int num_bags, OutT* __restrict__ out) {
    constexpr int GPB = 256 / L8;
    const int r = threadIdx.x % L8;
    const int64_t b = static_cast<int64_t>(blockIdx.x) * GPB + threadIdx.x / L8;
    if (b >= num_bags) return;  // whole groups leave together
    const int lo = bag_offsets[b], hi = bag_offsets[b + 1];
    const int chunks = dim / 8;
    float4 acc[NV8][2];
#pragma unroll
    for (int v = 0; v < NV8; ++v) acc[v][0] = acc[v][1] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int gl = __lane_id() & ~(L8 - 1);
    for (int base = lo; base < hi; base += L8) {
        const int j = base + r;
        int64_t row_off = 0;
        if (j < hi) row_off = lookup_row(list_keys, idx, j) * static_cast<int64_t>(dim) * 2;
        const int off_lo = static_cast<int>(row_off & 0xFFFFFFFFll), off_hi = static_cast<int>(row_off >> 32);
        const int cnt = hi - base < L8 ? hi - base : L8;
        for (int k0 = 0; k0 < cnt; k0 += kFwdUnroll) {
            uint4 x[kFwdUnroll][NV8];
#pragma unroll
            for (int q = 0; q < kFwdUnroll; ++q) {
                const bool on = k0 + q < cnt;  // uniform inside the group; k0 + q < L8 always (L8 >= kFwdUnroll)
                const uint32_t lo32 = static_cast<uint32_t>(__shfl(off_lo, gl + k0 + q, kWave));
                const uint32_t hi32 = static_cast<uint32_t>(__shfl(off_hi, gl + k0 + q, kWave));
                const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(table) +
                                                                  ((static_cast<uint64_t>(hi32) << 32) | lo32));
#pragma unroll
                for (int v = 0; v < NV8; ++v) {
                    const int c = r + v * L8;
                    x[q][v] = (on && c < chunks) ? src[c] : make_uint4(0u, 0u, 0u, 0u);
                }
            }
#pragma unroll
            for (int q = 0; q < kFwdUnroll; ++q) {
#pragma unroll
                for (int v = 0; v < NV8; ++v) {  // rows that were not loaded are zeros
                    float4 a, c;
                    widen8(table, x[q][v], a, c);
                    acc[v][0].x += a.x;
                    acc[v][0].y += a.y;
                    acc[v][0].z += a.z;
                    acc[v][0].w += a.w;
                    acc[v][1].x += c.x;
                    acc[v][1].y += c.y;
                    acc[v][1].z += c.z;
                    acc[v][1].w += c.w;
                }
            }
        }
    }
    float scale = 1.f;
    if (MEAN && hi > lo) scale = 1.f / static_cast<float>(hi - lo);
#pragma unroll
    for (int v = 0; v < NV8; ++v) {
        const int c = r + v * L8;
        if (c < chunks) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float4 a = acc[v][h];
                if (MEAN) {
                    a.x *= scale;
                    a.y *= scale;
                    a.z *= scale;
                    a.w *= scale;
                }
                store_words(out + static_cast<size_t>(b) * dim + c * 8 + h * 4, a);
            }
        }
    }
}

template <int L8, int NV8, typename TabT>
void fwd_pool_x8_launch(const TabT* table, int dim, const int64_t* list_keys, const int32_t* idx, const int32_t* bag_offsets,
                            int num_bags, int mode, int out_dtype, void* out, hipStream_t stream) {
    constexpr int GPB = 256 / L8;
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(num_bags) + GPB - 1) / GPB);
    const bool mean = mode == NP_POOL_MEAN;
    if (out_dtype == NP_BF16) {
        if (mean)
            NP_LAUNCH("fwd_pool", (fwd_pool_x8_kernel<L8, NV8, true, uint16_t, TabT>), dim3(grid), dim3(256), 0, stream, table, dim,
                      list_keys, idx, bag_offsets, num_bags, static_cast<uint16_t*>(out));
        else
            NP_LAUNCH("fwd_pool", (fwd_pool_x8_kernel<L8, NV8, false, uint16_t, TabT>), dim3(grid), dim3(256), 0, stream, table, dim,
                      list_keys, idx, bag_offsets, num_bags, static_cast<uint16_t*>(out));
    } else {
        if (mean)
            NP_LAUNCH("fwd_pool", (fwd_pool_x8_kernel<L8, NV8, true, float, TabT>), dim3(grid), dim3(256), 0, stream, table, dim,
                      list_keys, idx, bag_offsets, num_bags, static_cast<float*>(out));
        else
            NP_LAUNCH("fwd_pool", (fwd_pool_x8_kernel<L8, NV8, false, float, TabT>), dim3(grid), dim3(256), 0, stream, table, dim,
                      list_keys, idx, bag_offsets, num_bags, static_cast<float*>(out));
    }
}

#ifndef NP_SEQ_PER_GROUP
#define NP_SEQ_PER_GROUP 4
#endif
constexpr int kSeqPerGroup = NP_SEQ_PER_GROUP;  // output positions per group, their slot -> key -> row chains in flight together

// Resolves the wave's output positions once, one lane each (position -> bag -> slot -> key), and hands every
// group the byte offsets of its SPG rows by shuffle; -1 marks padding or a position past the end.
// ELEM_BYTES is the size of a table element.  All 64 lanes call it.
template <int LANES, int SPG, int ELEM_BYTES>
__device__ __forceinline__ void seq_row_offsets(int64_t wq0, int64_t total, int max_len, int dim, const int64_t* __restrict__ list_keys,
                                                const int32_t* __restrict__ idx, const int32_t* __restrict__ bag_offsets,
                                                int64_t (&off)[SPG]) {
    constexpr int PW = (kWave / LANES) * SPG;  // positions per wave
    static_assert(PW <= kWave, "one lane per position");
    const int lane = __lane_id();
    int64_t my_off = -1;
    if (lane < PW && wq0 + lane < total) {
        const int64_t q = wq0 + lane;
        const int b = static_cast<int>(static_cast<uint32_t>(q) / static_cast<uint32_t>(max_len));  // total < 2^31
        const int p = static_cast<int>(q - static_cast<int64_t>(b) * max_len);
        const int lo = bag_offsets[b];
        if (p < bag_offsets[b + 1] - lo) {
            const int j = lo + p;
            my_off = lookup_row(list_keys, idx, j) * static_cast<int64_t>(dim) * ELEM_BYTES;
        }
    }
    const int off_lo = static_cast<int>(my_off & 0xFFFFFFFFll), off_hi = static_cast<int>(my_off >> 32);
#pragma unroll
    for (int k = 0; k < SPG; ++k) {
        const int from = (lane / LANES) * SPG + k;
        const uint32_t lo32 = static_cast<uint32_t>(__shfl(off_lo, from, kWave));
        const int32_t hi32 = __shfl(off_hi, from, kWave);
        off[k] = (static_cast<int64_t>(hi32) << 32) | lo32;
    }
}

template <int LPR, int NV, typename OutT, typename TabT>
__global__ void __launch_bounds__(256)
fwd_seq_kernel(const TabT* __restrict__ table, int dim, const int64_t* __restrict__ list_keys, const int32_t* __restrict__ idx,
               const int32_t* __restrict__ bag_offsets, int num_bags, int max_len, OutT* __restrict__ out) {
    constexpr int GPB = 256 / LPR;
    constexpr int SPG = kSeqPerGroup < LPR ? kSeqPerGroup : LPR;  // positions per group; at most 64 per wave
    const int r = threadIdx.x % LPR;
    const int64_t total = static_cast<int64_t>(num_bags) * max_len;
    const int64_t q0 = (static_cast<int64_t>(blockIdx.x) * GPB + threadIdx.x / LPR) * SPG;  // first output position of the group
    const int64_t wq0 = (static_cast<int64_t>(blockIdx.x) * GPB + (threadIdx.x / kWave) * (kWave / LPR)) * SPG;  // ... of the wave
    const int words = dim / 4;
    int64_t off[SPG];
    seq_row_offsets<LPR, SPG, static_cast<int>(sizeof(TabT))>(wq0, total, max_len, dim, list_keys, idx, bag_offsets, off);
    float4 x[SPG][NV];
#pragma unroll
    for (int k = 0; k < SPG; ++k) {
        const TabT* src = reinterpret_cast<const TabT*>(reinterpret_cast<const char*>(table) + (off[k] < 0 ? 0 : off[k]));
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int wv = r + v * LPR;
            x[k][v] = (off[k] >= 0 && wv < words) ? load_word(src, wv) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
#pragma unroll
    for (int k = 0; k < SPG; ++k) {
        const int64_t q = q0 + k;
        if (q < total) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int wv = r + v * LPR;
                if (wv < words) store_words(out + static_cast<size_t>(q) * dim + wv * 4, x[k][v]);
            }
        }
    }
}

// Sequence output in bf16 for rows whose width is a multiple of 8: a lane owns 8 consecutive floats (two
// 16-byte loads) and writes them as 8 bf16 with one 16-byte store, so loads and stores are both full width.
// L8 lanes share a row (dim / 8 rounded up to a power of two, at most 64), NV8 chunks of 8 floats per lane.
// A block owns kSeqBlockPos consecutive output positions.  First every thread
// resolves several positions at once (position -> bag -> slot -> key -> row offset, all lanes busy, the chains of
// one thread in flight together) into LDS; then the groups stream over the block's positions, kSeqBatch rows per
// group in flight, reading each row offset from LDS.  The resolve phase of one block overlaps the copy phase of the
// others on the same CU.
#ifndef NP_SEQ_BLOCK_POS
#define NP_SEQ_BLOCK_POS 1024
#endif
constexpr int kSeqBlockPos = NP_SEQ_BLOCK_POS;
constexpr int kSeqBatch = 4;

template <int L8, int NV8>
__global__ void __launch_bounds__(256)
fwd_seq_bf16x8_kernel(const float* __restrict__ table, int dim, const int64_t* __restrict__ list_keys,
                             const int32_t* __restrict__ idx, const int32_t* __restrict__ bag_offsets, int num_bags, int max_len,
                             uint16_t* __restrict__ out) {
    constexpr int GPB = 256 / L8;
    static_assert(kSeqBlockPos % (GPB * kSeqBatch) == 0 && kSeqBlockPos % 256 == 0, "whole batches per block");
    __shared__ int64_t soff[kSeqBlockPos];
    const int64_t total = static_cast<int64_t>(num_bags) * max_len;
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kSeqBlockPos;
#pragma unroll
    for (int s = 0; s < kSeqBlockPos / 256; ++s) {
        const int64_t q = base + s * 256 + threadIdx.x;
        int64_t off = -1;  // padding or past the end
        if (q < total) {
            const int b = static_cast<int>(static_cast<uint32_t>(q) / static_cast<uint32_t>(max_len));  // total < 2^31
            const int p = static_cast<int>(q - static_cast<int64_t>(b) * max_len);
            const int lo = bag_offsets[b];
            if (p < bag_offsets[b + 1] - lo) off = lookup_row(list_keys, idx, lo + p) * static_cast<int64_t>(dim) * 4;
        }
        soff[s * 256 + threadIdx.x] = off;
    }
    __syncthreads();
    const int r = threadIdx.x % L8, g = threadIdx.x / L8;
    const int chunks = dim / 8;
    for (int i0 = g; i0 < kSeqBlockPos; i0 += GPB * kSeqBatch) {
        if (base + i0 >= total) break;  // later positions of this group are further out still
        float4 x[kSeqBatch][NV8][2];
#pragma unroll
        for (int u = 0; u < kSeqBatch; ++u) {
            const int64_t off = soff[i0 + u * GPB];
            const float4* src = reinterpret_cast<const float4*>(reinterpret_cast<const char*>(table) + (off < 0 ? 0 : off));
#pragma unroll
            for (int v = 0; v < NV8; ++v) {
                const int c = r + v * L8;
                const bool on = off >= 0 && c < chunks;
                x[u][v][0] = on ? src[2 * c] : make_float4(0.f, 0.f, 0.f, 0.f);
                x[u][v][1] = on ? src[2 * c + 1] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
#pragma unroll
        for (int u = 0; u < kSeqBatch; ++u) {
            const int64_t q = base + i0 + u * GPB;
            if (q < total) {
#pragma unroll
                for (int v = 0; v < NV8; ++v) {
                    const int c = r + v * L8;
                    if (c < chunks) {
                        const float4 a = x[u][v][0], b = x[u][v][1];
                        uint4 o;
                        o.x = static_cast<uint32_t>(f32_to_bf16(a.x)) | (static_cast<uint32_t>(f32_to_bf16(a.y)) << 16);
                        o.y = static_cast<uint32_t>(f32_to_bf16(a.z)) | (static_cast<uint32_t>(f32_to_bf16(a.w)) << 16);
                        o.z = static_cast<uint32_t>(f32_to_bf16(b.x)) | (static_cast<uint32_t>(f32_to_bf16(b.y)) << 16);
                        o.w = static_cast<uint32_t>(f32_to_bf16(b.z)) | (static_cast<uint32_t>(f32_to_bf16(b.w)) << 16);
                        store_stream(reinterpret_cast<uint4*>(out + static_cast<size_t>(q) * dim + c * 8), o);
                    }
                }
            }
        }
    }
}

template <int L8, int NV8>
void fwd_seq_bf16x8_launch(const float* table, int dim, const int64_t* list_keys, const int32_t* idx, const int32_t* bag_offsets,
                           int num_bags, int max_len, uint16_t* out, hipStream_t stream) {
    const int64_t total = static_cast<int64_t>(num_bags) * max_len;
    const unsigned grid = static_cast<unsigned>((total + kSeqBlockPos - 1) / kSeqBlockPos);
    NP_LAUNCH("fwd_seq", (fwd_seq_bf16x8_kernel<L8, NV8>), dim3(grid), dim3(256), 0, stream, table, dim, list_keys, idx,
              bag_offsets, num_bags, max_len, out);
}

template <int LPR, int NV, typename TabT>
__global__ void __launch_bounds__(256)
fwd_rows_kernel(const TabT* __restrict__ table, int dim, const int64_t* __restrict__ list_keys,
                const int32_t* __restrict__ d_num_list, int cap, TabT* __restrict__ rows_out) {
    constexpr int GPB = 256 / LPR;
    const int r = threadIdx.x % LPR;
    const int words = dim / 4;
    const int L = device_count(d_num_list, cap);
    for (int64_t p = static_cast<int64_t>(blockIdx.x) * GPB + threadIdx.x / LPR; p < L; p += static_cast<int64_t>(gridDim.x) * GPB) {
        const TabT* src = table + static_cast<size_t>(list_keys[p]) * dim;
        TabT* dst = rows_out + static_cast<size_t>(p) * dim;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int wv = r + v * LPR;
            if (wv < words) copy_word_stream(src, dst, wv);
        }
    }
}

struct FwdArgs {
    const void* table;
    int dim;
    const int64_t* list_keys;
    const int32_t* d_num_list;
    int cap;
    const int32_t* idx;
    const int32_t* bag_offsets;
    int num_bags, mode, max_len, out_dtype;
    void* out;
    void* rows_out;
    hipStream_t stream;
};

template <int LPR, int NV, typename TabT>
void fwd_launch(const FwdArgs& a) {
    constexpr int GPB = 256 / LPR;
    const TabT* table = static_cast<const TabT*>(a.table);
    if (a.num_bags > 0) {
        if (a.mode == NP_SEQ) {
            constexpr int SPG = kSeqPerGroup < LPR ? kSeqPerGroup : LPR;
            const int64_t total = static_cast<int64_t>(a.num_bags) * a.max_len;
            const int64_t per_block = static_cast<int64_t>(GPB) * SPG;
            const unsigned grid = static_cast<unsigned>((total + per_block - 1) / per_block);
            if (a.out_dtype == NP_BF16)
                NP_LAUNCH("fwd_seq", (fwd_seq_kernel<LPR, NV, uint16_t, TabT>), dim3(grid), dim3(256), 0, a.stream, table, a.dim,
                          a.list_keys, a.idx, a.bag_offsets, a.num_bags, a.max_len, static_cast<uint16_t*>(a.out));
            else
                NP_LAUNCH("fwd_seq", (fwd_seq_kernel<LPR, NV, float, TabT>), dim3(grid), dim3(256), 0, a.stream, table, a.dim,
                          a.list_keys, a.idx, a.bag_offsets, a.num_bags, a.max_len, static_cast<float*>(a.out));
        } else {
            const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(a.num_bags) + GPB - 1) / GPB);
            const bool mean = a.mode == NP_POOL_MEAN;
            if (a.out_dtype == NP_BF16) {
                if (mean)
                    NP_LAUNCH("fwd_pool", (fwd_pool_kernel<LPR, NV, true, uint16_t, TabT>), dim3(grid), dim3(256), 0, a.stream, table,
                              a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, static_cast<uint16_t*>(a.out));
                else
                    NP_LAUNCH("fwd_pool", (fwd_pool_kernel<LPR, NV, false, uint16_t, TabT>), dim3(grid), dim3(256), 0, a.stream, table,
                              a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, static_cast<uint16_t*>(a.out));
            } else {
                if (mean)
                    NP_LAUNCH("fwd_pool", (fwd_pool_kernel<LPR, NV, true, float, TabT>), dim3(grid), dim3(256), 0, a.stream, table,
                              a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, static_cast<float*>(a.out));
                else
                    NP_LAUNCH("fwd_pool", (fwd_pool_kernel<LPR, NV, false, float, TabT>), dim3(grid), dim3(256), 0, a.stream, table,
                              a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, static_cast<float*>(a.out));
            }
        }
    }
    if (a.rows_out && a.cap > 0) {
        int64_t want = (static_cast<int64_t>(a.cap) + GPB - 1) / GPB;
        const unsigned grid = static_cast<unsigned>(want < 16384 ? want : 16384);
        NP_LAUNCH("fwd_rows", (fwd_rows_kernel<LPR, NV, TabT>), dim3(grid), dim3(256), 0, a.stream, table, a.dim, a.list_keys,
                  a.d_num_list, a.cap, static_cast<TabT*>(a.rows_out));
    }
}

template <typename TabT>
void fwd_dispatch(const FwdArgs& a) {
    const int words = a.dim / 4;
    if (words <= 4) fwd_launch<4, 1, TabT>(a);
    else if (words <= 8) fwd_launch<8, 1, TabT>(a);
    else if (words <= 16) fwd_launch<16, 1, TabT>(a);
    else if (words <= 32) fwd_launch<32, 1, TabT>(a);
    else if (words <= 64) fwd_launch<64, 1, TabT>(a);
    else if (words <= 128) fwd_launch<64, 2, TabT>(a);
    else fwd_launch<64, 4, TabT>(a);
}

// A table of 16-bit elements: the full-width pooled route where the row shape allows, the generic kernels otherwise
// (sequence mode, narrow or odd rows, and the optional rows_out copy).
template <typename TabT>
void fwd_16bit(FwdArgs a, const TabT* t) {
    if (a.mode != NP_SEQ && a.dim % 8 == 0 && a.dim >= 32 && a.num_bags > 0 && aligned(t, 16)) {
        const int chunks = a.dim / 8;
        if (chunks <= 4) fwd_pool_x8_launch<4, 1>(t, a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, a.mode, a.out_dtype, a.out, a.stream);
        else if (chunks <= 8) fwd_pool_x8_launch<8, 1>(t, a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, a.mode, a.out_dtype, a.out, a.stream);
        else if (chunks <= 16) fwd_pool_x8_launch<16, 1>(t, a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, a.mode, a.out_dtype, a.out, a.stream);
        else if (chunks <= 32) fwd_pool_x8_launch<32, 1>(t, a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, a.mode, a.out_dtype, a.out, a.stream);
        else if (chunks <= 64) fwd_pool_x8_launch<64, 1>(t, a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, a.mode, a.out_dtype, a.out, a.stream);
        else fwd_pool_x8_launch<64, 2>(t, a.dim, a.list_keys, a.idx, a.bag_offsets, a.num_bags, a.mode, a.out_dtype, a.out, a.stream);
        a.num_bags = 0;  // what remains for the generic launcher is rows_out
    }
    fwd_dispatch<TabT>(a);
}

}  // namespace np

extern "C" {

size_t np_lookup_fwd_workspace_bytes(int32_t, int32_t, int32_t, int32_t) { return 0; }

int np_lookup_fwd_t(const void* table, int32_t table_dtype, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                    const int32_t* d_num_list, int32_t cap, const int32_t* idx, const int32_t* bag_offsets,
                    int32_t num_bags, int32_t n, int32_t mode, int32_t max_len, int32_t out_dtype, void* out,
                    void* rows_out, void* ws, size_t ws_bytes, void* stream) {
    (void)ws;
    (void)ws_bytes;
    if (!table || num_rows < 1 || num_bags < 0 || n < 0 || cap < 0 || !bag_offsets) return NP_ERR_INVALID_ARG;
    if (table_dtype != NP_F32 && table_dtype != NP_BF16 && table_dtype != NP_F16) return NP_ERR_INVALID_ARG;
    if (mode != NP_POOL_SUM && mode != NP_POOL_MEAN && mode != NP_SEQ) return NP_ERR_INVALID_ARG;
    if (out_dtype != NP_F32 && out_dtype != NP_BF16) return NP_ERR_INVALID_ARG;
    if (mode == NP_SEQ && max_len < 1) return NP_ERR_INVALID_ARG;
    if (dim < 4 || dim % 4 != 0 || dim > NP_MAX_DIM) return NP_ERR_UNSUPPORTED;
    if ((num_bags > 0 && !out) || (n > 0 && !list_keys && !idx)) return NP_ERR_INVALID_ARG;
    if (rows_out && (!d_num_list || !list_keys)) return NP_ERR_INVALID_ARG;
    const size_t row_align = table_dtype == NP_F32 ? 16 : 8;
    if (!np::aligned(table, row_align) || !np::aligned(out, out_dtype == NP_BF16 ? 8 : 16) || !np::aligned(rows_out, row_align))
        return NP_ERR_INVALID_ARG;
    if (mode == NP_SEQ && static_cast<int64_t>(num_bags) * max_len > INT32_MAX) return NP_ERR_UNSUPPORTED;
    np::FwdArgs a{table, dim, list_keys, d_num_list, cap, idx, bag_offsets, num_bags, mode, max_len, out_dtype, out, rows_out,
                  static_cast<hipStream_t>(stream)};
    if (table_dtype == NP_BF16) {
        np::fwd_16bit<uint16_t>(a, static_cast<const uint16_t*>(table));
        return np::launch_status();
    }
    if (table_dtype == NP_F16) {
        np::fwd_16bit<__half>(a, static_cast<const __half*>(table));
        return np::launch_status();
    }
    if (mode == NP_SEQ && out_dtype == NP_BF16 && dim % 8 == 0 && num_bags > 0 && np::aligned(out, 16)) {
        // full-width route for bf16 sequences; the optional rows_out copy still goes through the generic launcher
        hipStream_t st = static_cast<hipStream_t>(stream);
        uint16_t* o = static_cast<uint16_t*>(out);
        const float* t = static_cast<const float*>(table);
        const int chunks = dim / 8;
        if (chunks <= 4) np::fwd_seq_bf16x8_launch<4, 1>(t, dim, list_keys, idx, bag_offsets, num_bags, max_len, o, st);
        else if (chunks <= 8) np::fwd_seq_bf16x8_launch<8, 1>(t, dim, list_keys, idx, bag_offsets, num_bags, max_len, o, st);
        else if (chunks <= 16) np::fwd_seq_bf16x8_launch<16, 1>(t, dim, list_keys, idx, bag_offsets, num_bags, max_len, o, st);
        else if (chunks <= 32) np::fwd_seq_bf16x8_launch<32, 1>(t, dim, list_keys, idx, bag_offsets, num_bags, max_len, o, st);
        else if (chunks <= 64) np::fwd_seq_bf16x8_launch<64, 1>(t, dim, list_keys, idx, bag_offsets, num_bags, max_len, o, st);
        else np::fwd_seq_bf16x8_launch<64, 2>(t, dim, list_keys, idx, bag_offsets, num_bags, max_len, o, st);
        a.num_bags = 0;  // pooled / sequence part done; what remains for the generic launcher is rows_out
    }
    np::fwd_dispatch<float>(a);
    return np::launch_status();
}

int np_lookup_fwd(const float* table, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                  const int32_t* d_num_list, int32_t cap, const int32_t* idx, const int32_t* bag_offsets,
                  int32_t num_bags, int32_t n, int32_t mode, int32_t max_len, int32_t out_dtype, void* out,
                  float* rows_out, void* ws, size_t ws_bytes, void* stream) {
    return np_lookup_fwd_t(table, NP_F32, num_rows, dim, list_keys, d_num_list, cap, idx, bag_offsets, num_bags, n, mode,
                           max_len, out_dtype, out, rows_out, ws, ws_bytes, stream);
}

}  // extern "C"
