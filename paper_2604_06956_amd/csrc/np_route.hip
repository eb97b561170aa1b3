// np_route: stable bucketing of the distinct keys by owner shard into the packed layout a key All2All
// sends (Section IV-A, "Key Routing": deduplicated keys are partitioned into buckets following the
// table-sharding rule).  One partition pass with digit = shard(key); the per-shard totals of that pass
// are the split counts and their prefix sums the send offsets.
#include "np_partition.hpp"

namespace np {

struct RoutePolicy {
    using KeyT = int64_t;
    static constexpr bool kStageDigit = true;
    const int64_t* unique;
    int64_t* send_keys;
    int32_t* send_from_unique;
    int32_t* unique_to_send;
    FastMod fm;
    int hash;
    __device__ __forceinline__ int64_t load_key(int64_t i) const { return unique[i]; }
    __device__ __forceinline__ void load(int64_t i, int64_t& k, uint32_t& v) const {
        k = unique[i];
        v = static_cast<uint32_t>(i);
    }
    __device__ __forceinline__ uint32_t digit(int64_t k) const {
        const uint64_t x = hash ? mix64(static_cast<uint64_t>(k)) : static_cast<uint64_t>(k);
        return fastmod64(x, fm);
    }
    __device__ __forceinline__ void store(uint32_t dst, int64_t k, uint32_t v) const {
        send_keys[dst] = k;
        send_from_unique[dst] = static_cast<int32_t>(v);
    }
    __device__ __forceinline__ void placed(int64_t i, uint32_t dst) const { unique_to_send[i] = static_cast<int32_t>(dst); }
};

__global__ void __launch_bounds__(256)
route_compose_kernel(const int32_t* __restrict__ inverse, int n, const int32_t* __restrict__ unique_to_send,
                     int32_t* __restrict__ lookup_to_send) {
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; j < n;
         j += static_cast<int64_t>(gridDim.x) * blockDim.x)
        lookup_to_send[j] = unique_to_send[inverse[j]];
}

// The allocation-free variant keeps its scratch (the chunk x shard histogram matrix and the per-shard totals) in this
// file-scope device array instead of a caller workspace.  In host code the array's name is only a handle: its device
// address is asked for once per device with hipGetSymbolAddress and kept in route_scratch_ptr.
constexpr size_t kRouteStaticHistBytes = sizeof(uint32_t) * static_cast<size_t>(kTargetChunks) * NP_ROUTE_STATIC_MAX_SHARDS;
constexpr size_t kRouteStaticBytes = kRouteStaticHistBytes + sizeof(uint32_t) * NP_ROUTE_STATIC_MAX_SHARDS;
static __device__ __align__(256) unsigned char scratch[kRouteStaticBytes];

static std::atomic<unsigned char*> route_scratch_ptr[kMaxDevices];

// Device address of this device's copy of `scratch` (nullptr on failure).  The calling thread's current device decides
// which copy; racing first calls ask twice and store the same address.
static unsigned char* route_scratch_for_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    unsigned char* p = route_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) {
        (void)hipGetLastError();
        return nullptr;
    }
    p = static_cast<unsigned char*>(sym);
    route_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

static int route_check(const int64_t* unique, const int32_t* d_num_unique, int32_t cap, int32_t num_shards, int32_t shard_fn,
                       int64_t* send_keys, int32_t* splits, int32_t* send_offsets, int32_t* send_from_unique,
                       int32_t* unique_to_send, const int32_t* inverse, int32_t n, int32_t* lookup_to_send, int32_t max_shards) {
    if (cap < 0 || num_shards < 1 || !d_num_unique || !splits || !send_offsets) return NP_ERR_INVALID_ARG;
    if (shard_fn != NP_SHARD_MOD && shard_fn != NP_SHARD_HASH) return NP_ERR_INVALID_ARG;
    if (cap > 0 && (!unique || !send_keys || !send_from_unique || !unique_to_send)) return NP_ERR_INVALID_ARG;
    if ((inverse == nullptr) != (lookup_to_send == nullptr) || n < 0) return NP_ERR_INVALID_ARG;
    if (num_shards > max_shards) return NP_ERR_UNSUPPORTED;
    if (!aligned(unique, 8) || !aligned(send_keys, 8)) return NP_ERR_INVALID_ARG;
    return NP_OK;
}

// Enqueues the pass; H holds part_hist_elems() words, bin_total num_shards words.  Both are fully written before they
// are read (every chunk writes every bin of its histogram row), so neither has to be cleared.
static int route_enqueue(const int64_t* unique, const int32_t* d_num_unique, int32_t cap, int32_t num_shards, int32_t shard_fn,
                         int64_t* send_keys, int32_t* splits, int32_t* send_offsets, int32_t* send_from_unique,
                         int32_t* unique_to_send, const int32_t* inverse, int32_t n, int32_t* lookup_to_send, uint32_t* H,
                         uint32_t* bin_total, hipStream_t s) {
    const ChunkPlan plan = make_chunk_plan(cap);
    int nbits = 0;
    while ((1 << nbits) < num_shards) ++nbits;
    RoutePolicy pol{unique, send_keys, send_from_unique, unique_to_send, make_fastmod(static_cast<uint32_t>(num_shards)),
                    shard_fn == NP_SHARD_HASH ? 1 : 0};
    run_partition_pass(pol, cap, d_num_unique, num_shards, nbits, plan, H, bin_total, splits, send_offsets, s, "route_hist",
                       "route_colscan", "route_scatter");
    if (inverse && n > 0) {
        int grid = (n + 255) / 256;
        if (grid > 8192) grid = 8192;
        NP_LAUNCH("route_compose", route_compose_kernel, dim3(grid), dim3(256), 0, s, inverse, n, unique_to_send, lookup_to_send);
    }
    return launch_status();
}

}  // namespace np

extern "C" {

size_t np_route_workspace_bytes(int32_t cap, int32_t num_shards) {
    if (cap < 0 || num_shards < 1 || num_shards > NP_MAX_SHARDS) return 0;
    const np::ChunkPlan plan = np::make_chunk_plan(cap);
    return np::align_up(4 * np::part_hist_elems(plan, num_shards), 256) + np::align_up(4 * static_cast<size_t>(num_shards), 256);
}

int np_route(const int64_t* unique, const int32_t* d_num_unique, int32_t cap, int32_t num_shards, int32_t shard_fn,
             int64_t* send_keys, int32_t* splits, int32_t* send_offsets, int32_t* send_from_unique,
             int32_t* unique_to_send, const int32_t* inverse, int32_t n, int32_t* lookup_to_send, void* ws,
             size_t ws_bytes, void* stream) {
    const int rc = np::route_check(unique, d_num_unique, cap, num_shards, shard_fn, send_keys, splits, send_offsets, send_from_unique,
                                   unique_to_send, inverse, n, lookup_to_send, NP_MAX_SHARDS);
    if (rc != NP_OK) return rc;
    if (!ws || !np::aligned(ws, 256) || ws_bytes < np_route_workspace_bytes(cap, num_shards)) return NP_ERR_WORKSPACE;
    np::WsCursor cur(ws);
    uint32_t* H = cur.take<uint32_t>(np::part_hist_elems(np::make_chunk_plan(cap), num_shards));
    uint32_t* bin_total = cur.take<uint32_t>(num_shards);
    return np::route_enqueue(unique, d_num_unique, cap, num_shards, shard_fn, send_keys, splits, send_offsets, send_from_unique,
                             unique_to_send, inverse, n, lookup_to_send, H, bin_total, static_cast<hipStream_t>(stream));
}

int np_route_static(const int64_t* unique, const int32_t* d_num_unique, int32_t cap, int32_t num_shards, int32_t shard_fn,
                    int64_t* send_keys, int32_t* splits, int32_t* send_offsets, int32_t* send_from_unique,
                    int32_t* unique_to_send, const int32_t* inverse, int32_t n, int32_t* lookup_to_send, void* stream) {
    const int rc = np::route_check(unique, d_num_unique, cap, num_shards, shard_fn, send_keys, splits, send_offsets, send_from_unique,
                                   unique_to_send, inverse, n, lookup_to_send, NP_ROUTE_STATIC_MAX_SHARDS);
    if (rc != NP_OK) return rc;
    unsigned char* base = np::route_scratch_for_current_device();
    if (!base) return NP_ERR_HIP;
    uint32_t* H = reinterpret_cast<uint32_t*>(base);
    uint32_t* bin_total = reinterpret_cast<uint32_t*>(base + np::kRouteStaticHistBytes);
    return np::route_enqueue(unique, d_num_unique, cap, num_shards, shard_fn, send_keys, splits, send_offsets, send_from_unique,
                             unique_to_send, inverse, n, lookup_to_send, H, bin_total, static_cast<hipStream_t>(stream));
}

}  // extern "C"
