// Shared host/device helpers of the gfx950 sparse-embedding library: launch bookkeeping, wave64
// primitives, the XCD-aware block mapping and the routing hash.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nestpipe.h"

namespace np {

constexpr int kWave = 64;
constexpr int kNumXcd = 8;  // MI355X: 8 accelerator dies, workgroup i is dispatched to die i % 8

// ---------------------------------------------------------------- host side -----------------------

// Thresholds that choose between two code paths with identical results (np_tune_set / np_tune_get at the C boundary).
enum Tunable { kTuneEmitOrderMinN = 0, kTuneBwdOrderMinDyBytes = 1, kTuneBwdRowIndex = 2, kTuneBwdSinglesByBag = 3, kTuneCount = 4 };
int64_t tune_get(Tunable which);

void prof_begin(const char* name, hipStream_t stream);
void prof_end(hipStream_t stream);

inline int launch_status() { return hipGetLastError() == hipSuccess ? NP_OK : NP_ERR_HIP; }

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of the caller's workspace.
struct WsCursor {
    char* base;
    size_t used;
    explicit WsCursor(void* p) : base(static_cast<char*>(p)), used(0) {}
    template <typename T>
    T* take(size_t count) {
        T* r = reinterpret_cast<T*>(base + used);
        used += align_up(count * sizeof(T), 256);
        return r;
    }
};

#define NP_LAUNCH(name, kernel, grid, block, shmem, stream, ...)                       \
    do {                                                                              \
        ::np::prof_begin(name, stream);                                               \
        hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);          \
        ::np::prof_end(stream);                                                       \
    } while (0)

// ---------------------------------------------------------------- device side ---------------------

// Logical block index such that consecutive logical blocks run on the same die (they then share one L2,
// so partial cache lines written by neighbours merge before they reach HBM).  A bijection on [0, nblocks).
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
    const int q = nblocks / kNumXcd, r = nblocks % kNumXcd;
    const int x = bid % kNumXcd, i = bid / kNumXcd;
    return x * q + (x < r ? x : r) + i;
}

__device__ __forceinline__ uint64_t lanemask_lt() {
    const int l = __lane_id();
    return l == 0 ? 0ull : (~0ull >> (64 - l));
}

// A count the device holds (distinct keys, list entries, pairs), never more than the host bound `cap` that the buffers and
// the grid were sized for and never negative: a stale or corrupt count must not make a kernel walk past its buffers.
__device__ __forceinline__ int device_count(const int32_t* __restrict__ d_count, int cap) {
    const int v = *d_count;
    return v < 0 ? 0 : (v < cap ? v : cap);
}

// Routing hash (a bijection of 64-bit words): odd multiplier, xor-shift, twice.
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t k) {
    const uint64_t C = 0x9E3779B97F4A7C15ull;
    uint64_t a = k * C;
    a ^= a >> 32;
    a *= C;
    a ^= a >> 29;
    return a;
}

// x mod s for s < 2^16 through a precomputed reciprocal: magic = floor(2^32 / s).
struct FastMod {
    uint32_t s, magic, pow32;  // pow32 = 2^32 mod s
};

inline FastMod make_fastmod(uint32_t s) {
    FastMod f;
    f.s = s;
    f.magic = s == 1 ? 0xFFFFFFFFu : static_cast<uint32_t>((1ull << 32) / s);
    f.pow32 = static_cast<uint32_t>((1ull << 32) % s);
    return f;
}

__device__ __forceinline__ uint32_t fastmod32(uint32_t x, const FastMod& f) {
    uint32_t q = __umulhi(x, f.magic);
    uint32_t r = x - q * f.s;
    while (r >= f.s) r -= f.s;
    return r;
}

__device__ __forceinline__ uint32_t fastmod64(uint64_t x, const FastMod& f) {
    const uint32_t hi = fastmod32(static_cast<uint32_t>(x >> 32), f);
    const uint32_t lo = fastmod32(static_cast<uint32_t>(x), f);
    return fastmod32(hi * f.pow32 + lo, f);  // hi, pow32 < 2^16: the product fits in 32 bits
}

// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS traffic, not for global loads
// still in flight (a plain __syncthreads drains those too, which serialises every prefetch behind the barrier).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Keeps the compiler from moving memory accesses across this point; emits no instruction.
__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }

__device__ __forceinline__ int wave_incl_scan(int v) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int t = __shfl_up(v, d, kWave);
        if (static_cast<int>(__lane_id()) >= d) v += t;
    }
    return v;
}

// s_waitcnt vmcnt(0) with the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt
// 11:8): every global load and store this wave has issued is complete.
__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Exclusive scan of one int per thread over a block of NW waves.  `smem` holds NW + 1 ints.  Returns the
// exclusive prefix; *total receives the block sum.  Contains two LDS barriers.
template <int NW>
__device__ __forceinline__ int block_excl_scan(int v, int* smem, int* total) {
    const int w = threadIdx.x / kWave;
    const int inc = wave_incl_scan(v);
    lds_barrier();  // smem may still be read from a previous call
    if (__lane_id() == kWave - 1) smem[w] = inc;
    lds_barrier();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const int s = smem[i];
        if (i < w) base += s;
        tot += s;
    }
    *total = tot;
    return base + inc - v;
}

// Accesses to data that is touched once per launch (index streams, output rows): marked non-temporal so that
// they leave L2 first and the rows that are gathered again and again stay.  Only for whole rows and coalesced
// streams: scattered 4- and 8-byte stores rely on L2 to merge partial lines and get much slower with the hint.
#ifndef NP_STREAM_HINTS
#define NP_STREAM_HINTS 1
#endif
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void store_stream(float4* p, const float4& a) {
#if NP_STREAM_HINTS
    f32x4_t v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t*>(p));
#else
    *p = a;
#endif
}

__device__ __forceinline__ void store_stream(uint2* p, const uint2& a) {
#if NP_STREAM_HINTS
    u32x2_t v = {a.x, a.y};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x2_t*>(p));
#else
    *p = a;
#endif
}

__device__ __forceinline__ float4 load_stream(const float4* p) {
#if NP_STREAM_HINTS
    const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
#else
    return *p;
#endif
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store_stream(uint4* p, const uint4& a) {
#if NP_STREAM_HINTS
    u32x4_t v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p));
#else
    *p = a;
#endif
}

template <typename T>
__device__ __forceinline__ T load_stream(const T* p) {
#if NP_STREAM_HINTS
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

// fp32 -> bf16, round to nearest even; NaN becomes a quiet NaN.
__device__ __forceinline__ uint16_t f32_to_bf16(float x) {
    uint32_t b = __float_as_uint(x);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((b >> 16) | 0x0040u);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return static_cast<uint16_t>(b >> 16);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(static_cast<uint32_t>(h) << 16); }

// A row "word" is four consecutive elements: 16 bytes of an fp32 row, 8 bytes of a bf16 row.  Reading a bf16 word
// widens exactly; writing one rounds to nearest even.
__device__ __forceinline__ float4 load_word(const float* row, int w) { return reinterpret_cast<const float4*>(row)[w]; }

__device__ __forceinline__ float4 load_word(const uint16_t* row, int w) {
    const uint2 u = reinterpret_cast<const uint2*>(row)[w];
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                       __uint_as_float(u.y & 0xFFFF0000u));
}

__device__ __forceinline__ uint2 pack_bf16x4(const float4& a) {
    uint2 o;
    o.x = static_cast<uint32_t>(f32_to_bf16(a.x)) | (static_cast<uint32_t>(f32_to_bf16(a.y)) << 16);
    o.y = static_cast<uint32_t>(f32_to_bf16(a.z)) | (static_cast<uint32_t>(f32_to_bf16(a.w)) << 16);
    return o;
}

__device__ __forceinline__ void store_word_stream(float* row, int w, const float4& a) {
    store_stream(reinterpret_cast<float4*>(row) + w, a);
}

__device__ __forceinline__ void store_word_stream(uint16_t* row, int w, const float4& a) {
    store_stream(reinterpret_cast<uint2*>(row) + w, pack_bf16x4(a));
}

// fp16 rows are typed __half (bf16 rows are uint16_t): same 8-byte words, hardware conversions (nearest even).
__device__ __forceinline__ float4 load_word(const __half* row, int w) {
    const uint2 u = reinterpret_cast<const uint2*>(row)[w];
    const __half2 lo = *reinterpret_cast<const __half2*>(&u.x), hi = *reinterpret_cast<const __half2*>(&u.y);
    return make_float4(__low2float(lo), __high2float(lo), __low2float(hi), __high2float(hi));
}

// fp32 -> fp16, nearest even, of a value that has already been rounded to fp32.  The empty asm pins the fp32 value in
// a register: without it the compiler may merge the producing fp32 multiply or subtract with the conversion into
// one mixed-precision instruction that rounds the exact result once, which differs from the two-step result on
// double-rounding ties.
__device__ __forceinline__ __half f32_to_f16(float x) {
    asm volatile("" : "+v"(x));
    return __float2half_rn(x);
}

__device__ __forceinline__ void store_word_stream(__half* row, int w, const float4& a) {
    const __half2 lo = __halves2half2(f32_to_f16(a.x), f32_to_f16(a.y));
    const __half2 hi = __halves2half2(f32_to_f16(a.z), f32_to_f16(a.w));
    uint2 o;
    o.x = *reinterpret_cast<const uint32_t*>(&lo);
    o.y = *reinterpret_cast<const uint32_t*>(&hi);
    store_stream(reinterpret_cast<uint2*>(row) + w, o);
}

__device__ __forceinline__ void copy_word_stream(const __half* src, __half* dst, int w) {
    store_stream(reinterpret_cast<uint2*>(dst) + w, reinterpret_cast<const uint2*>(src)[w]);
}

// Bit copy of one word (no conversion, so NaN payloads survive).
__device__ __forceinline__ void copy_word_stream(const float* src, float* dst, int w) {
    store_stream(reinterpret_cast<float4*>(dst) + w, reinterpret_cast<const float4*>(src)[w]);
}

__device__ __forceinline__ void copy_word_stream(const uint16_t* src, uint16_t* dst, int w) {
    store_stream(reinterpret_cast<uint2*>(dst) + w, reinterpret_cast<const uint2*>(src)[w]);
}

// Row-wise Adagrad pieces shared by np_sparse_adagrad and the fused backward: written with explicit fused
// multiply-adds so that both kernels round identically whatever the compiler would contract on its own.
__device__ __forceinline__ float sumsq4(const float4& g) { return fmaf(g.w, g.w, fmaf(g.z, g.z, fmaf(g.y, g.y, g.x * g.x))); }

__device__ __forceinline__ float adagrad_state(float s_old, float sumsq, float inv_dim) { return fmaf(sumsq, inv_dim, s_old); }

__device__ __forceinline__ void adagrad_step4(float4& w, const float4& g, float lr, float denom) {
    w.x -= (lr * g.x) / denom;
    w.y -= (lr * g.y) / denom;
    w.z -= (lr * g.z) / denom;
    w.w -= (lr * g.w) / denom;
}

}  // namespace np
