// Host-side odds and ends of the library (version, status text, per-kernel event timing) and the two
// harness kernels: the stateless table initialiser and the plain copy used as a bandwidth yardstick.
#include <atomic>
#include <cstring>
#include <string>
#include <vector>

#include "np_common.hpp"

namespace np {

namespace {
struct ProfRecord {
    const char* name;
    hipEvent_t start, stop;
};
bool g_prof_on = false;
std::vector<ProfRecord> g_prof_log;                       // records of the current collection window
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_prof_pool;  // events created so far, reused
size_t g_prof_next = 0;
std::vector<std::string> g_prof_only;                     // when not empty: only launches with these names are timed
}  // namespace

namespace {
struct TunableSpec {
    const char* name;
    int64_t initial, lo, hi;
};
// initial values: where each alternative starts to pay on an MI355X (the measurements are in the kernels' comments)
const TunableSpec kTunables[kTuneCount] = {
    {"emit_order_min_n", int64_t(1) << 22, 0, INT64_MAX},          // np_dedup: lookups from which the inverse map is written tile-ordered
    {"bwd_order_min_dy_bytes", int64_t(256) << 20, 0, INT64_MAX},  // np_lookup_bwd: upstream-gradient bytes from which tiles run locality-ordered
    {"bwd_row_index", 0, 0, 1},  // np_lookup_bwd: 1 = resolve the upstream-gradient row of every sorted position in a pass of its own
    {"bwd_singles_by_bag", 0, 0, 1},  // np_lookup_bwd: 1 = keys with one lookup are copied bag by bag, the reduction skips them
};
std::atomic<int64_t> g_tune[kTuneCount] = {{kTunables[0].initial}, {kTunables[1].initial}, {kTunables[2].initial},
                                           {kTunables[3].initial}};
}  // namespace

int64_t tune_get(Tunable which) { return g_tune[which].load(std::memory_order_relaxed); }

void prof_begin(const char* name, hipStream_t stream) {
    if (!g_prof_on) return;
    if (!g_prof_only.empty()) {
        bool wanted = false;
        for (const std::string& w : g_prof_only) wanted |= w == name;
        if (!wanted) return;
    }
    if (g_prof_next == g_prof_pool.size()) {
        hipEvent_t a = nullptr, b = nullptr;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
            (void)hipGetLastError();
            return;
        }
        g_prof_pool.emplace_back(a, b);
    }
    auto& ev = g_prof_pool[g_prof_next];
    g_prof_log.push_back({name, ev.first, ev.second});
    (void)hipEventRecord(ev.first, stream);
}

void prof_end(hipStream_t stream) {
    if (!g_prof_on || g_prof_log.size() != g_prof_next + 1) return;
    (void)hipEventRecord(g_prof_log.back().stop, stream);
    ++g_prof_next;
}

// ---------------------------------------------------------------- harness kernels -----------------

// Initial value of table element e (row * dim + column): a hash of e and the seed mapped to [-0.01, 0.01).
__device__ __forceinline__ float table_init_value(uint64_t e, uint64_t seed_term) {
    uint64_t h = e + seed_term;
    h ^= h >> 31;
    h *= 0xD6E8FEB86659FD93ull;
    h ^= h >> 27;
    h *= 0xA3B195354A39B70Dull;
    h ^= h >> 33;
    const int q = static_cast<int>(h >> 40) - 8388608;
    return static_cast<float>(q) * (0.01f / 8388608.0f);
}

// What a value reads back as after being stored in a table of the given element type.
__device__ __forceinline__ float as_stored(const float*, float v) { return v; }
__device__ __forceinline__ float as_stored(const uint16_t*, float v) { return bf16_to_f32(f32_to_bf16(v)); }
__device__ __forceinline__ float as_stored(const __half*, float v) { return __half2float(f32_to_f16(v)); }

// TabT = float: the value itself; uint16_t: rounded to bf16; __half: rounded to fp16 (nearest even).
template <typename TabT>
__global__ void __launch_bounds__(256) table_init_kernel(TabT* __restrict__ table, uint64_t num_words, uint64_t seed_term) {
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
    for (uint64_t w = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; w < num_words; w += stride) {
        float v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = table_init_value(w * 4 + c, seed_term);
        store_word_stream(table + w * 4, 0, make_float4(v[0], v[1], v[2], v[3]));
    }
}

__global__ void zero_u64_kernel(unsigned long long* p) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0ull;
}

// One thread per row (test harness code: simplicity over speed); integer atomics only.
template <typename TabT>
__global__ void __launch_bounds__(256)
table_count_changed_kernel(const TabT* __restrict__ table, uint64_t num_rows, int words_per_row, uint64_t seed_term,
                           unsigned long long* __restrict__ count) {
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
    unsigned long long local = 0;
    for (uint64_t row = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; row < num_rows; row += stride) {
        bool changed = false;
        for (int wq = 0; wq < words_per_row && !changed; ++wq) {
            const uint64_t w = row * words_per_row + wq;
            const float4 t = load_word(table + w * 4, 0);
            const float got[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float v = table_init_value(w * 4 + c, seed_term);
                v = as_stored(static_cast<const TabT*>(nullptr), v);
                changed |= __float_as_uint(v) != __float_as_uint(got[c]);
            }
        }
        local += changed ? 1ull : 0ull;
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) local += __shfl_xor(local, d, kWave);
    if (__lane_id() == 0 && local) atomicAdd(count, local);
}

// Precondition check of a batch: integer atomics on four counters, one pass.
__global__ void __launch_bounds__(256)
check_batch_kernel(const int64_t* __restrict__ keys, int n, int64_t num_rows, const int32_t* __restrict__ bag_offsets, int num_bags,
                   unsigned long long* __restrict__ errors) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    unsigned long long bad_keys = 0, bad_steps = 0;
    if (keys)
        for (int64_t i = t0; i < n; i += stride) {
            const int64_t k = keys[i];
            bad_keys += (k < 0 || k >= num_rows) ? 1ull : 0ull;
        }
    if (bag_offsets) {
        for (int64_t b = t0; b < num_bags; b += stride) bad_steps += bag_offsets[b + 1] < bag_offsets[b] ? 1ull : 0ull;
        if (t0 == 0) {
            if (bag_offsets[0] != 0) atomicAdd(errors + 2, 1ull);
            if (bag_offsets[num_bags] != n) atomicAdd(errors + 3, 1ull);
        }
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        bad_keys += __shfl_xor(bad_keys, d, kWave);
        bad_steps += __shfl_xor(bad_steps, d, kWave);
    }
    if (__lane_id() == 0) {
        if (bad_keys) atomicAdd(errors + 0, bad_keys);
        if (bad_steps) atomicAdd(errors + 1, bad_steps);
    }
}

__global__ void zero_u64x4_kernel(unsigned long long* p) {
    if (blockIdx.x == 0 && threadIdx.x < 4) p[threadIdx.x] = 0ull;
}

// The bandwidth yardstick: every block streams one contiguous slab, four 16-byte loads in flight per thread, streaming
// hints on both sides.  Measured on this GPU for 2 GiB: 5.6 TB/s (read + write) against 4.5-5.0 TB/s for a plain
// grid-stride loop; a read-only pass of the same shape reaches 6.5 TB/s, a write-only one 5.8 TB/s.
__global__ void __launch_bounds__(256) stream_copy_kernel(float4* __restrict__ dst, const float4* __restrict__ src, uint64_t num_words) {
    constexpr int kInFlight = 4;
    const uint64_t per = (num_words + gridDim.x - 1) / gridDim.x;
    const uint64_t lo = per * blockIdx.x;
    const uint64_t hi = lo + per < num_words ? lo + per : num_words;
    uint64_t w = lo + threadIdx.x;
    for (; w + (kInFlight - 1) * 256 < hi; w += kInFlight * 256) {
        float4 x[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) x[u] = load_stream(src + w + u * 256);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) store_stream(dst + w + u * 256, x[u]);
    }
    for (; w < hi; w += 256) store_stream(dst + w, load_stream(src + w));
}

// Yardstick for the row kernels: random gathers of whole rows of 64 floats (16 lanes x 16 bytes, eight rows in flight per
// lane group, the access pattern of np_lookup_fwd / np_lookup_bwd), summed in groups of 64 so that next to nothing is
// written.  rows[i] = (a hash of i) mod num_rows: the working set is num_rows * 256 bytes.
__global__ void __launch_bounds__(256)
gather_rate_kernel(const float4* __restrict__ src, uint32_t num_rows, int64_t n, uint32_t seed, float4* __restrict__ out) {
    constexpr int LPR = 16, UN = 8;
    const int r = threadIdx.x % LPR;
    const int64_t g = static_cast<int64_t>(blockIdx.x) * (256 / LPR) + threadIdx.x / LPR;
    const int64_t base = g * 64;
    if (base >= n) return;
    const int gl = __lane_id() & ~(LPR - 1);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c = 0; c < 64; c += LPR) {
        uint32_t h = static_cast<uint32_t>(base + c + r) * 2654435761u + seed;
        h ^= h >> 16; h *= 0x7feb352dU; h ^= h >> 15; h *= 0x846ca68bU; h ^= h >> 16;
        const uint32_t mine = static_cast<uint32_t>((static_cast<uint64_t>(h) * num_rows) >> 32);
        for (int k0 = 0; k0 < LPR; k0 += UN) {
            float4 x[UN];
#pragma unroll
            for (int q = 0; q < UN; ++q) {
                const uint32_t row = static_cast<uint32_t>(__shfl(static_cast<int>(mine), gl + k0 + q, kWave));
                x[q] = src[static_cast<uint64_t>(row) * LPR + r];
            }
#pragma unroll
            for (int q = 0; q < UN; ++q) {
                acc.x += x[q].x;
                acc.y += x[q].y;
                acc.z += x[q].z;
                acc.w += x[q].w;
            }
        }
    }
    out[g * LPR + r] = acc;
}

}  // namespace np

extern "C" {

int np_tune_set(const char* name, int64_t value) {
    if (!name) return NP_ERR_INVALID_ARG;
    for (int i = 0; i < np::kTuneCount; ++i) {
        if (std::strcmp(name, np::kTunables[i].name) == 0) {
            if (value < np::kTunables[i].lo || value > np::kTunables[i].hi) return NP_ERR_INVALID_ARG;
            np::g_tune[i].store(value, std::memory_order_relaxed);
            return NP_OK;
        }
    }
    return NP_ERR_INVALID_ARG;
}

int64_t np_tune_get(const char* name) {
    if (!name) return -1;
    for (int i = 0; i < np::kTuneCount; ++i)
        if (std::strcmp(name, np::kTunables[i].name) == 0) return np::g_tune[i].load(std::memory_order_relaxed);
    return -1;
}

int np_version(void) { return 10301; }  // 1.3.1: same interface as 1.3.0 (np_route_static, np_tune_set / np_tune_get); sort passes on (key, position) pairs

const char* np_status_string(int status) {
    switch (status) {
        case NP_OK: return "ok";
        case NP_ERR_INVALID_ARG: return "invalid argument";
        case NP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case NP_ERR_UNSUPPORTED: return "unsupported configuration";
        case NP_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int np_util_table_init_t(void* table, int32_t table_dtype, int64_t num_rows, int32_t dim, uint64_t seed, void* stream) {
    if (table_dtype != NP_F32 && table_dtype != NP_BF16 && table_dtype != NP_F16) return NP_ERR_INVALID_ARG;
    if (!table || num_rows < 0 || dim < 4 || dim % 4 != 0 || !np::aligned(table, table_dtype == NP_F32 ? 16 : 8))
        return NP_ERR_INVALID_ARG;
    const uint64_t words = static_cast<uint64_t>(num_rows) * static_cast<uint64_t>(dim) / 4;
    if (words == 0) return NP_OK;
    const uint64_t want = (words + 255) / 256;
    const unsigned grid = static_cast<unsigned>(want < 65536 ? want : 65536);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t seed_term = seed * 0x2545F4914F6CDD1Dull;
    if (table_dtype == NP_BF16)
        NP_LAUNCH("table_init", np::table_init_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, static_cast<uint16_t*>(table), words,
                  seed_term);
    else if (table_dtype == NP_F16)
        NP_LAUNCH("table_init", np::table_init_kernel<__half>, dim3(grid), dim3(256), 0, s, static_cast<__half*>(table), words, seed_term);
    else
        NP_LAUNCH("table_init", np::table_init_kernel<float>, dim3(grid), dim3(256), 0, s, static_cast<float*>(table), words, seed_term);
    return np::launch_status();
}

int np_util_table_init(float* table, int64_t num_rows, int32_t dim, uint64_t seed, void* stream) {
    return np_util_table_init_t(table, NP_F32, num_rows, dim, seed, stream);
}

int np_util_table_count_changed_t(const void* table, int32_t table_dtype, int64_t num_rows, int32_t dim, uint64_t seed,
                                  unsigned long long* d_count, void* stream) {
    if (table_dtype != NP_F32 && table_dtype != NP_BF16 && table_dtype != NP_F16) return NP_ERR_INVALID_ARG;
    if (!table || !d_count || num_rows < 0 || dim < 4 || dim % 4 != 0 || !np::aligned(table, table_dtype == NP_F32 ? 16 : 8))
        return NP_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    NP_LAUNCH("zero_u64", np::zero_u64_kernel, dim3(1), dim3(64), 0, s, d_count);
    if (num_rows > 0) {
        const uint64_t want = (static_cast<uint64_t>(num_rows) + 255) / 256;
        const unsigned grid = static_cast<unsigned>(want < 65536 ? want : 65536);
        const uint64_t seed_term = seed * 0x2545F4914F6CDD1Dull;
        if (table_dtype == NP_BF16)
            NP_LAUNCH("table_count_changed", np::table_count_changed_kernel<uint16_t>, dim3(grid), dim3(256), 0, s,
                      static_cast<const uint16_t*>(table), static_cast<uint64_t>(num_rows), dim / 4, seed_term, d_count);
        else if (table_dtype == NP_F16)
            NP_LAUNCH("table_count_changed", np::table_count_changed_kernel<__half>, dim3(grid), dim3(256), 0, s,
                      static_cast<const __half*>(table), static_cast<uint64_t>(num_rows), dim / 4, seed_term, d_count);
        else
            NP_LAUNCH("table_count_changed", np::table_count_changed_kernel<float>, dim3(grid), dim3(256), 0, s,
                      static_cast<const float*>(table), static_cast<uint64_t>(num_rows), dim / 4, seed_term, d_count);
    }
    return np::launch_status();
}

int np_util_table_count_changed(const float* table, int64_t num_rows, int32_t dim, uint64_t seed,
                                unsigned long long* d_count, void* stream) {
    return np_util_table_count_changed_t(table, NP_F32, num_rows, dim, seed, d_count, stream);
}

int np_util_check_batch(const int64_t* keys, int32_t n, int64_t num_rows, const int32_t* bag_offsets, int32_t num_bags,
                        unsigned long long* d_errors, void* stream) {
    if (n < 0 || num_bags < 0 || num_rows < 0 || !d_errors || (n > 0 && !keys) || (num_bags > 0 && !bag_offsets))
        return NP_ERR_INVALID_ARG;
    if (!np::aligned(keys, 8) || !np::aligned(bag_offsets, 4) || !np::aligned(d_errors, 8)) return NP_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    NP_LAUNCH("check_zero", np::zero_u64x4_kernel, dim3(1), dim3(64), 0, s, d_errors);
    const int64_t work = n > num_bags ? n : num_bags;
    if (work == 0) return np::launch_status();
    int64_t want = (work + 255) / 256;
    const unsigned grid = static_cast<unsigned>(want < 8192 ? want : 8192);
    NP_LAUNCH("check_batch", np::check_batch_kernel, dim3(grid), dim3(256), 0, s, n > 0 ? keys : nullptr, n, num_rows,
              num_bags > 0 ? bag_offsets : nullptr, num_bags, d_errors);
    return np::launch_status();
}

int np_util_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || bytes % 16 != 0 || !np::aligned(dst, 16) || !np::aligned(src, 16)) return NP_ERR_INVALID_ARG;
    const uint64_t words = bytes / 16;
    if (words == 0) return NP_OK;
    const uint64_t want = (words + 255) / 256;
    const unsigned grid = static_cast<unsigned>(want < 16384 ? want : 16384);
    NP_LAUNCH("stream_copy", np::stream_copy_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
              static_cast<float4*>(dst), static_cast<const float4*>(src), words);
    return np::launch_status();
}

int np_util_gather_rate(const float* src, int64_t num_rows, int64_t n, uint32_t seed, float* out, void* stream) {
    if (!src || !out || num_rows < 1 || num_rows > 0xFFFFFFFFll || n < 0 || n % 64 != 0) return NP_ERR_INVALID_ARG;
    if (!np::aligned(src, 16) || !np::aligned(out, 16)) return NP_ERR_INVALID_ARG;
    if (n == 0) return NP_OK;
    const int64_t blocks = (n / 64 + 15) / 16;
    if (blocks > 0x7FFFFFFFll) return NP_ERR_UNSUPPORTED;
    NP_LAUNCH("gather_rate", np::gather_rate_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, static_cast<hipStream_t>(stream),
              reinterpret_cast<const float4*>(src), static_cast<uint32_t>(num_rows), n, seed, reinterpret_cast<float4*>(out));
    return np::launch_status();
}

int np_prof_enable(int on) {
    np::g_prof_on = on != 0;
    np::g_prof_log.clear();
    np::g_prof_next = 0;
    return NP_OK;
}

int np_prof_only(const char* names) {
    np::g_prof_only.clear();
    if (!names) return NP_OK;
    std::string cur;
    for (const char* p = names;; ++p) {
        if (*p == ',' || *p == '\0') {
            if (!cur.empty()) np::g_prof_only.push_back(cur);
            cur.clear();
            if (*p == '\0') break;
        } else {
            cur.push_back(*p);
        }
    }
    return NP_OK;
}

int np_prof_collect(const char** names, float* ms, int max_entries) {
    int count = 0;
    for (size_t i = 0; i < np::g_prof_next && count < max_entries; ++i) {
        auto& r = np::g_prof_log[i];
        float t = 0.f;
        if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess) {
            (void)hipGetLastError();
            t = -1.f;
        }
        if (names) names[count] = r.name;
        if (ms) ms[count] = t;
        ++count;
    }
    np::g_prof_log.clear();
    np::g_prof_next = 0;
    return count;
}

}  // extern "C"
