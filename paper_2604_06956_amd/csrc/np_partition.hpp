// Stable multi-way partition of a sequence by a small integer "digit", the building block of both the
// radix sort inside np_dedup (digit = a bit field of the key) and the bucketing of np_route (digit =
// owner shard).  Three kernels per pass, no inter-block waiting:
//
//   part_hist     one block per chunk: LDS histogram of the chunk's digits           -> H[chunk][bin]
//   part_colscan  exclusive scan of every column of H over the chunks (in place)      -> binTotal[bin]
//   part_scatter  one block per chunk, tile by tile: every item gets its stable rank among the items of its wave with
//                 the same digit (lane masks collected in LDS, ballots for the digit's upper bits), per-bin prefix sums
//                 over the waves and the bins give its slot, the tile is reordered through LDS and written out in runs
//
// A chunk is a run of consecutive tiles owned by one block, sized so that at most kTargetChunks blocks
// cover the input: all of them are resident at once, the same number on every CU (no tail round), and the
// histogram matrix stays small.
// The scatter kernel maps chunks to blocks so that neighbouring chunks run on the same die: the short
// runs they append to each bin then merge in that die's L2 instead of reaching HBM as partial lines.
#pragma once

#include <atomic>

#include "np_common.hpp"

namespace np {

#ifndef NP_PART_THREADS
#define NP_PART_THREADS 512
#endif
#ifndef NP_PART_IPT
#define NP_PART_IPT 8
#endif
constexpr int kPartThreads = NP_PART_THREADS;
constexpr int kPartWaves = kPartThreads / kWave;
constexpr int kPartIPT = NP_PART_IPT;
constexpr int kPartTile = kPartThreads * kPartIPT;
static_assert(kPartIPT * kWave <= 65535, "per-wave digit counters are 16 bits wide");
// The 16-bit per-wave counters of one bin lie side by side and are scanned through one wide LDS access per kCntRowWaves waves.
constexpr int kCntRowWaves = kPartWaves % 8 == 0 ? 8 : 4;
static_assert(kPartWaves % kCntRowWaves == 0, "the per-wave 16-bit counters of one bin fill whole 8- or 16-byte words");
struct __align__(kCntRowWaves * 2) CntRow {
    uint32_t w[kCntRowWaves / 2];
};
constexpr int kPartMaxBins = 4096;
#ifndef NP_TARGET_CHUNKS
#define NP_TARGET_CHUNKS 512  // two blocks on each of the 256 CUs: 384, 640, 768 and 1024 leave a ragged last round
#endif
constexpr int kTargetChunks = NP_TARGET_CHUNKS;
constexpr int kMaxDevices = 64;  // devices whose dynamic-LDS opt-in is remembered
constexpr int kColscanThreads = 1024;
constexpr int kHistThreads = 1024;

// The input is cut into whole tiles, the tiles into num_chunks runs that differ by at most one tile, so that the
// number of blocks is exactly the target whenever there are that many tiles.
struct ChunkPlan {
    int num_chunks;
    int num_tiles;  // tiles of kPartTile items
};

inline ChunkPlan make_chunk_plan(int64_t cap) {
    int64_t tiles = (cap + kPartTile - 1) / kPartTile;
    if (tiles < 1) tiles = 1;
    ChunkPlan p;
    p.num_chunks = static_cast<int>(tiles < kTargetChunks ? tiles : kTargetChunks);
    p.num_tiles = static_cast<int>(tiles);
    return p;
}

// First item of chunk c (c = num_chunks gives the end of the last chunk).
__host__ __device__ __forceinline__ int64_t chunk_begin(const ChunkPlan& p, int c) {
    return (static_cast<int64_t>(c) * p.num_tiles / p.num_chunks) * kPartTile;
}

// Words reserved for the histogram matrix: sized for the largest chunk count so that the workspace
// requirement grows monotonically with the input size (the chunk count itself does not).
inline size_t part_hist_elems(const ChunkPlan&, int bins) { return static_cast<size_t>(kTargetChunks) * bins; }

// gofs, binstart, btot (one word per bin each) and 16 words of scan scratch, rounded up so that the staging area
// behind them is 16-byte aligned for any bin count (64-bit keys are staged there).
__host__ __device__ __forceinline__ size_t part_fixed_lds_bytes(int bins) {
    return (3 * sizeof(uint32_t) * static_cast<size_t>(bins) + 64 + 15) / 16 * 16;
}

// The low kMaskBits bits of a digit are matched through a per-wave table of 64-bit lane masks in LDS (one OR, one read and
// one clearing write per item) instead of one ballot per bit; only the bits above them are matched with ballots.
#ifndef NP_PART_MASK_BITS
#define NP_PART_MASK_BITS 8
#endif
constexpr int kMaskBits = NP_PART_MASK_BITS;
constexpr int kMaskSlots = 1 << kMaskBits;

__host__ __device__ __forceinline__ size_t part_cnt_bytes(int bins) {  // per-wave digit counters, 16-byte rounded
    return (sizeof(uint16_t) * kPartWaves * static_cast<size_t>(bins) + 15) / 16 * 16;
}

__host__ __device__ __forceinline__ size_t part_rank_bytes(int bins) {  // counters and, behind them, the lane-mask tables
    return part_cnt_bytes(bins) + (kMaskBits > 0 ? sizeof(unsigned long long) * kPartWaves * kMaskSlots : 0);
}

template <typename KeyT>
inline size_t part_stage_bytes(bool stage_digit) {
    return (sizeof(KeyT) + sizeof(uint32_t) + (stage_digit ? sizeof(uint16_t) : 0)) * kPartTile;
}

// The staging area of the reordered tile gets LDS of its own when two blocks per CU still fit (fewer barriers per tile:
// the counters of the next tile are cleared while this one is staged); otherwise it shares the counters' storage.
#ifndef NP_PART_LDS_PER_BLOCK
#define NP_PART_LDS_PER_BLOCK (80 * 1024)  // half of a CU's 160 KB
#endif
constexpr size_t kPartLdsPerBlock = NP_PART_LDS_PER_BLOCK;
template <typename KeyT>
inline bool part_stage_aliased(int bins, bool stage_digit) {
    return part_fixed_lds_bytes(bins) + part_rank_bytes(bins) + part_stage_bytes<KeyT>(stage_digit) > kPartLdsPerBlock;
}

template <typename KeyT>
inline size_t part_scatter_lds_bytes(int bins, bool stage_digit) {
    const size_t fixed = part_fixed_lds_bytes(bins);
    const size_t rank = part_rank_bytes(bins);  // a wave ranks kPartIPT * 64 <= 65535 items
    const size_t stage = part_stage_bytes<KeyT>(stage_digit);
    if (!part_stage_aliased<KeyT>(bins, stage_digit)) return fixed + rank + stage;
    return fixed + (rank > stage ? rank : stage);
}

// The counters of bin d lie side by side, wave w at column w ^ (cnt_swizzle(d) << 1): without the swizzle the lanes of one
// wave, which differ in d only, would all fall into a quarter of the LDS banks.
constexpr int kCntSwzShift = kPartWaves >= 16 ? 2 : (kPartWaves == 8 ? 3 : 4);
constexpr int kCntSwzMask = kCntRowWaves / 2 - 1;
__device__ __forceinline__ uint32_t cnt_swizzle(uint32_t d) { return (d >> kCntSwzShift) & kCntSwzMask; }
__device__ __forceinline__ uint32_t cnt_index(uint32_t d, int w) { return d * kPartWaves + (static_cast<uint32_t>(w) ^ (cnt_swizzle(d) << 1)); }
__device__ __forceinline__ void cnt_row_permute(CntRow& x, uint32_t swz) {  // its own inverse
    if (kCntRowWaves == 8) {
        if (swz & 1u) {
            uint32_t t = x.w[0]; x.w[0] = x.w[1]; x.w[1] = t;
            t = x.w[2 % (kCntRowWaves / 2)]; x.w[2 % (kCntRowWaves / 2)] = x.w[3 % (kCntRowWaves / 2)]; x.w[3 % (kCntRowWaves / 2)] = t;
        }
        if (swz & 2u) {
            uint32_t t = x.w[0]; x.w[0] = x.w[2 % (kCntRowWaves / 2)]; x.w[2 % (kCntRowWaves / 2)] = t;
            t = x.w[1]; x.w[1] = x.w[3 % (kCntRowWaves / 2)]; x.w[3 % (kCntRowWaves / 2)] = t;
        }
    } else if (swz & 1u) {
        const uint32_t t = x.w[0]; x.w[0] = x.w[1]; x.w[1] = t;
    }
}

// Lanes of the wave holding the same digit as this lane (only lanes with valid == true take part).
__device__ __forceinline__ uint64_t match_any(uint32_t d, int nbits, bool valid) {
    uint64_t peers = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (d >> b) & 1u;
        const uint64_t bal = __ballot(bit);
        peers &= bit ? bal : ~bal;
    }
    return peers;
}

// The item count the kernels work on: the device-side count when one is given, never more than the host bound the
// buffers and the grid were sized for (a stale or corrupt count must not walk past them).
__device__ __forceinline__ int64_t part_count(int n_host, const int* __restrict__ d_n) {
    return d_n ? device_count(d_n, n_host) : n_host;
}

// A policy supplies:
//   using KeyT; static constexpr bool kStageDigit;
//   __device__ void load(int64_t i, KeyT& k, uint32_t& v) const;   item i of the input
//   __device__ KeyT load_key(int64_t i) const;
//   __device__ uint32_t digit(KeyT k) const;
//   __device__ void store(uint32_t dst, KeyT k, uint32_t v) const; item placed at output slot dst
//   __device__ void placed(int64_t i, uint32_t dst) const;         input item i went to dst (may be a no-op)

// A streaming read with one LDS add per run: it runs with kHistThreads threads per block, twice the scatter
// kernel's, to keep enough loads in flight with two blocks per CU (0.21 -> 0.19 ms for three passes).
template <class P>
__global__ void __launch_bounds__(kHistThreads)
part_hist_kernel(P pol, int n_host, const int* __restrict__ d_n, int bins, ChunkPlan plan, uint32_t* __restrict__ H) {
    extern __shared__ uint32_t lh[];
    const int c = blockIdx.x;
    const int64_t n = part_count(n_host, d_n);
    for (int b = threadIdx.x; b < bins; b += kHistThreads) lh[b] = 0;
    __syncthreads();
    const int64_t lo = chunk_begin(plan, c);
    int64_t hi = chunk_begin(plan, c + 1);
    if (hi > n) hi = n;
    constexpr int kBatch = 8;  // independent loads in flight per thread
    const int lane = threadIdx.x % kWave;
    // the next batch is requested before the current one is counted (unconditional loads; past the end: the chunk's last
    // item, masked below)
    typename P::KeyT k[kBatch], kn[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) kn[q] = typename P::KeyT(0);
    if (lo < hi) {  // uniform
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            const int64_t i = lo + q * kHistThreads + threadIdx.x;
            kn[q] = pol.load_key(i < hi ? i : hi - 1);
        }
    }
    for (int64_t base = lo; base < hi; base += static_cast<int64_t>(kHistThreads) * kBatch) {
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            k[q] = kn[q];
            const int64_t i = base + static_cast<int64_t>(kHistThreads) * kBatch + q * kHistThreads + threadIdx.x;
            kn[q] = pol.load_key(i < hi ? i : hi - 1);
        }
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            // The lanes of a wave hold consecutive items, so the valid lanes are a prefix of the wave.  After the
            // first pass equal digits arrive in runs (a popular key fills whole waves): one add per run of equal
            // digits instead of one per lane keeps such waves from serialising on a single LDS address.
            const int64_t i = base + q * kHistThreads + threadIdx.x;
            const bool valid = i < hi;
            const uint32_t d = valid ? pol.digit(k[q]) : 0xFFFFFFFFu;
            const uint32_t dprev = __shfl_up(d, 1, kWave);
            const bool head = valid && (lane == 0 || d != dprev);
            const uint64_t heads = __ballot(head);
            const int num_valid = __popcll(__ballot(valid));
            if (head) {
                const uint64_t above = lane == kWave - 1 ? 0ull : (heads >> (lane + 1));
                const int run = above ? __builtin_ctzll(above) + 1 : num_valid - lane;
                atomicAdd(&lh[d], static_cast<uint32_t>(run));
            }
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < bins; b += kHistThreads) H[static_cast<size_t>(c) * bins + b] = lh[b];
}

// Block = 16 waves x 64 bins: wave y sums, then rewrites as exclusive prefixes, its slice of the chunks.
template <int THREADS>
__global__ void __launch_bounds__(THREADS)
part_colscan_kernel(uint32_t* __restrict__ H, int num_chunks, int bins, uint32_t* __restrict__ bin_total) {
    constexpr int NY = THREADS / kWave;
    __shared__ uint32_t part[NY][kWave];
    const int lane = threadIdx.x % kWave, y = threadIdx.x / kWave;
    const int bin = blockIdx.x * kWave + lane;
    const int per = (num_chunks + NY - 1) / NY;
    const int c0 = y * per;
    const int c1 = c0 + per < num_chunks ? c0 + per : num_chunks;
    uint32_t sum = 0;
    if (bin < bins) {
        for (int c = c0; c < c1; c += 8) {
            uint32_t t[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) t[q] = c + q < c1 ? H[static_cast<size_t>(c + q) * bins + bin] : 0u;
#pragma unroll
            for (int q = 0; q < 8; ++q) sum += t[q];
        }
    }
    part[y][lane] = sum;
    __syncthreads();
    uint32_t base = 0, total = 0;
#pragma unroll
    for (int yy = 0; yy < NY; ++yy) {
        const uint32_t s = part[yy][lane];
        if (yy < y) base += s;
        total += s;
    }
    if (bin < bins) {
        uint32_t run = base;
        for (int c = c0; c < c1; c += 8) {
            uint32_t t[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) t[q] = c + q < c1 ? H[static_cast<size_t>(c + q) * bins + bin] : 0u;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (c + q < c1) H[static_cast<size_t>(c + q) * bins + bin] = run;
                run += t[q];
            }
        }
        if (y == 0) bin_total[bin] = total;
    }
}

// One exclusive scan of an int per thread across the block with a single barrier inside; `smem` (kPartWaves ints) must not
// be in use by a previous call any more (here: several barriers lie between two calls).
__device__ __forceinline__ int part_block_scan(int v, int* smem, int* total) {
    const int w = threadIdx.x / kWave;
    const int inc = wave_incl_scan(v);
    if (__lane_id() == kWave - 1) smem[w] = inc;
    lds_barrier();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kPartWaves; ++i) {
        const int s = smem[i];
        if (i < w) base += s;
        tot += s;
    }
    *total = tot;
    return base + inc - v;
}

// What the kernel costs (three sort passes over 42 M items of a Zipf batch, 0.77 ms): with the stores redirected to
// consecutive addresses the passes take 0.50 ms, so a third of the time is the scattered stores, and they cost by their
// NUMBER, not their bytes: every run of items that a tile appends to a bin leaves the CU as a write of its own (uniformly
// random keys, four items per bin and tile: 0.70 ms for 63 M runs of 16 bytes; the 42 M single stores of np_dedup's inverse map
// cost the same per store).  Hence pairs instead of two arrays where a policy can (np_dedup's 32-bit keys: 0.90 -> 0.77 ms).
// The rest is the ranking: lane masks in LDS instead of ten ballots per item (0.95 -> 0.90 ms), the counters of a bin side by
// side and bank-swizzled, five barriers per tile instead of eight (no measurable change: the kernel is not bound by LDS).
// Measured and not taken: the digit width as a template argument so that the ballot loop unrolls (1.02 ms against 0.95),
// three blocks per CU instead of two by capping the kernel at 80 registers (amdgpu_waves_per_eu 6: the ranks and the
// prefetched tile no longer fit and spill, 1.80 ms with 768 chunks, 2.05 ms with 512), blocks of 256 threads, four per CU
// (tiles of 2048 items make the runs half as long: 1.13 ms against 0.90), blocks of 1024 threads, one per CU (tiles of 8192
// items: 0.75 ms against 0.77, and the counters of 4096 bins no longer fit), 10 or 12 items per thread (150 / 170
// registers: one block per CU).
template <class P, bool ALIAS>
__global__ void __launch_bounds__(kPartThreads)
part_scatter_kernel(P pol, int n_host, const int* __restrict__ d_n, int bins, int nbits, ChunkPlan plan,
                    const uint32_t* __restrict__ H, const uint32_t* __restrict__ bin_total,
                    int32_t* __restrict__ totals_out /* nullable: [bins] */, int32_t* __restrict__ offsets_out /* nullable: [bins+1] */) {
    using KeyT = typename P::KeyT;
    constexpr bool kPairs = sizeof(KeyT) == 4;  // 32-bit keys are staged side by side with their payload: one 8-byte access
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint32_t* gofs = reinterpret_cast<uint32_t*>(smem_raw);  // where the chunk's next item of every bin goes
    uint32_t* binstart = gofs + bins;                         // first slot of every bin in the reordered tile
    uint32_t* delta = binstart + bins;                        // the tile's count per bin, then gofs - binstart of this tile
    int* scan_tmp = reinterpret_cast<int*>(delta + bins);     // 16 ints
    unsigned char* un = smem_raw + part_fixed_lds_bytes(bins);
    // Per-wave digit counters [bins][waves] and, behind them, the per-wave lane-mask tables.  Plain (not volatile) accesses:
    // a volatile LDS access makes the compiler wait for every outstanding global load as well, which would drain the
    // prefetch of the next tile at the first counter access.  Where lanes of a wave hand values to each other through LDS, a
    // compiler-only fence keeps the accesses in program order; the wave's LDS operations execute in that order.
    uint16_t* cnt = reinterpret_cast<uint16_t*>(un);
    unsigned long long* wmask = reinterpret_cast<unsigned long long*>(un + part_cnt_bytes(bins)) + (threadIdx.x / kWave) * kMaskSlots;
    const unsigned long long lanebit = 1ull << (threadIdx.x % kWave);
    unsigned char* st = ALIAS ? un : un + part_rank_bytes(bins);
    KeyT* skey = reinterpret_cast<KeyT*>(st);
    uint32_t* sval = reinterpret_cast<uint32_t*>(skey + kPartTile);
    uint2* spair = reinterpret_cast<uint2*>(st);
    uint16_t* sdig = reinterpret_cast<uint16_t*>(st + (sizeof(KeyT) + sizeof(uint32_t)) * kPartTile);

    const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
    const int c = xcd_remap(blockIdx.x, gridDim.x);
    const int64_t n = part_count(n_host, d_n);
    const int bpt = (bins + kPartThreads - 1) / kPartThreads;
    const int b0 = tid * bpt;
    const int b1 = b0 + bpt < bins ? b0 + bpt : bins;
    const int zn = static_cast<int>(part_rank_bytes(bins) / 16);
    uint4* zero_from = reinterpret_cast<uint4*>(un);

    // global offset of this chunk's first item of every bin
    {
        int local = 0;
        for (int b = b0; b < b1; ++b) local += static_cast<int>(bin_total[b]);
        int total;
        int run = block_excl_scan<kPartWaves>(local, scan_tmp, &total);
        for (int b = b0; b < b1; ++b) {
            const uint32_t t = bin_total[b];
            gofs[b] = static_cast<uint32_t>(run) + H[static_cast<size_t>(c) * bins + b];
            if (c == 0 && totals_out) totals_out[b] = static_cast<int32_t>(t);
            if (c == 0 && offsets_out) offsets_out[b] = run;
            run += static_cast<int>(t);
        }
        if (c == 0 && offsets_out && tid == 0) offsets_out[bins] = total;
    }
    if (!ALIAS)
        for (int i = tid; i < zn; i += kPartThreads) zero_from[i] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();

    const int64_t lo = chunk_begin(plan, c);
    int64_t hi = chunk_begin(plan, c + 1);
    if (hi > n) hi = n;
    const uint64_t lt = lanemask_lt();

    // the items of the first tile; later tiles are fetched one iteration ahead and stay in flight across the LDS
    // barriers of the tile being ranked
    // Loads past the chunk's end are redirected to its last item instead of being skipped: unconditional loads are issued
    // back to back and stay in flight, conditional ones are waited for one by one.  What they bring is never used
    // (positions past tile_count are masked everywhere below).
    KeyT kn[kPartIPT];
    uint32_t vn[kPartIPT];
    const int64_t last = hi - 1;
#pragma unroll
    for (int i = 0; i < kPartIPT; ++i) {
        kn[i] = KeyT(0);
        vn[i] = 0;
    }
    if (lo < hi) {  // uniform
#pragma unroll
        for (int i = 0; i < kPartIPT; ++i) {
            const int64_t at = lo + w * (kWave * kPartIPT) + i * kWave + lane;
            pol.load(at < hi ? at : last, kn[i], vn[i]);
        }
    }

    for (int64_t tile_base = lo; tile_base < hi; tile_base += kPartTile) {
        const int tile_count = hi - tile_base < kPartTile ? static_cast<int>(hi - tile_base) : kPartTile;
        if (ALIAS) {  // the previous tile was staged where the counters and the mask tables live
            for (int i = tid; i < zn; i += kPartThreads) zero_from[i] = make_uint4(0u, 0u, 0u, 0u);
            lds_barrier();
        }

        KeyT k[kPartIPT];
        uint32_t v[kPartIPT], d[kPartIPT], r[kPartIPT];
#pragma unroll
        for (int i = 0; i < kPartIPT; ++i) {
            const int idx = w * (kWave * kPartIPT) + i * kWave + lane;
            k[i] = kn[i];
            v[i] = vn[i];
            d[i] = idx < tile_count ? pol.digit(k[i]) : 0;
        }
#pragma unroll
        for (int i = 0; i < kPartIPT; ++i) {
            const int64_t at = tile_base + kPartTile + w * (kWave * kPartIPT) + i * kWave + lane;
            pol.load(at < hi ? at : last, kn[i], vn[i]);
        }
        // stable rank of every item among the items of its wave with the same digit
#pragma unroll
        for (int i = 0; i < kPartIPT; ++i) {
            const int idx = w * (kWave * kPartIPT) + i * kWave + lane;
            const bool valid = idx < tile_count;
            uint16_t* ctr = cnt + cnt_index(d[i], w);
            uint64_t peers;
            unsigned long long* slot = wmask + (d[i] & (kMaskSlots - 1));
            // One digit in the whole wave (a popular key's run after the first pass, or few bins): every valid lane is a
            // peer, no table needed; 64 lanes would also serialise on one slot.
            const uint64_t vmask = __ballot(valid);
            const bool one_digit = __ballot(valid && d[i] == static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(d[i]))) == vmask;
            if (one_digit) {  // uniform
                peers = vmask;
            } else if (kMaskBits > 0) {
                // every lane sets its bit in the slot of its digit's low bits, then reads the slot back: the lanes whose
                // digits agree in those bits.  A wave's LDS operations execute in program order, so the read sees all 64
                // ORs; the lowest peer clears the slot for the next round.
                if (valid) atomicOr(slot, lanebit);
                compiler_fence();
                __builtin_amdgcn_wave_barrier();
                peers = *slot;
                if (nbits > kMaskBits) peers &= match_any(d[i] >> kMaskBits, nbits - kMaskBits, valid);
            } else {
                peers = match_any(d[i], nbits, valid);
            }
            const uint32_t pre = *ctr;
            const uint64_t below = peers & lt;
            r[i] = pre + __popcll(below);
            compiler_fence();
            __builtin_amdgcn_wave_barrier();
            if (valid && below == 0) {
                *ctr = static_cast<uint16_t>(pre + __popcll(peers));
                if (kMaskBits > 0 && !one_digit) *slot = 0;
            }
            compiler_fence();
            __builtin_amdgcn_wave_barrier();
        }
        lds_barrier();
        // per bin: exclusive scan over the waves, total of the tile: one wide read, the prefixes in registers, one wide write
        int local = 0;
        for (int b = b0; b < b1; ++b) {
            CntRow* row = reinterpret_cast<CntRow*>(cnt + b * kPartWaves);
            const uint32_t swz = cnt_swizzle(static_cast<uint32_t>(b));
            uint32_t s = 0;
#pragma unroll
            for (int q = 0; q < kPartWaves / kCntRowWaves; ++q) {
                CntRow x = row[q];
                cnt_row_permute(x, swz);
#pragma unroll
                for (int j = 0; j < kCntRowWaves / 2; ++j) {
                    const uint32_t lo16 = x.w[j] & 0xffffu, hi16 = x.w[j] >> 16;
                    x.w[j] = s | ((s + lo16) << 16);  // both prefixes stay below 65536 (a tile has fewer items)
                    s += lo16 + hi16;
                }
                cnt_row_permute(x, swz);
                row[q] = x;
            }
            delta[b] = s;
            local += static_cast<int>(s);
        }
        int total;
        int run = part_block_scan(local, scan_tmp, &total);
        for (int b = b0; b < b1; ++b) {
            const uint32_t t = delta[b], g = gofs[b];
            binstart[b] = static_cast<uint32_t>(run);
            delta[b] = g - static_cast<uint32_t>(run);  // slot p of the reordered tile goes to delta[bin] + p
            gofs[b] = g + t;
            run += static_cast<int>(t);
        }
        lds_barrier();
#pragma unroll
        for (int i = 0; i < kPartIPT; ++i) {
            const int idx = w * (kWave * kPartIPT) + i * kWave + lane;
            r[i] += binstart[d[i]] + static_cast<uint32_t>(cnt[cnt_index(d[i], w)]);  // position inside the reordered tile
            const uint32_t dst = delta[d[i]] + r[i];
            if (idx < tile_count && dst < static_cast<uint32_t>(n)) pol.placed(tile_base + idx, dst);
        }
        lds_barrier();  // the counters are dead from here on
        if (!ALIAS) {   // cleared for the next tile beside the staging; the mask tables are clear already (every round clears its slots)
            const int zc = static_cast<int>(part_cnt_bytes(bins) / 16);
            for (int i = tid; i < zc; i += kPartThreads) zero_from[i] = make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int i = 0; i < kPartIPT; ++i) {
            const int idx = w * (kWave * kPartIPT) + i * kWave + lane;
            if (idx < tile_count) {
                if constexpr (kPairs) {
                    spair[r[i]] = make_uint2(static_cast<uint32_t>(k[i]), v[i]);
                } else {
                    skey[r[i]] = k[i];
                    sval[r[i]] = v[i];
                }
                if (P::kStageDigit) sdig[r[i]] = static_cast<uint16_t>(d[i]);
            }
        }
        lds_barrier();
        for (int p = tid; p < tile_count; p += kPartThreads) {
            KeyT key;
            uint32_t val;
            if constexpr (kPairs) {
                const uint2 kv = spair[p];
                key = static_cast<KeyT>(kv.x);
                val = kv.y;
            } else {
                key = skey[p];
                val = sval[p];
            }
            const uint32_t dd = P::kStageDigit ? static_cast<uint32_t>(sdig[p]) : pol.digit(key);
            const uint32_t dst = delta[dd] + static_cast<uint32_t>(p);
            if (dst < static_cast<uint32_t>(n)) pol.store(dst, key, val);  // always true; keeps a broken histogram from writing out of bounds
        }
        // Aliased, the next tile clears the staging area at its top: wait for the readers.  Otherwise the next writes to
        // anything read above (delta, the staging area) lie behind the next tile's barriers.
        if (ALIAS) lds_barrier();
    }
}

// Enqueue one partition pass over n_host items, or over min(*d_n, n_host) items when d_n is given.  H needs
// part_hist_elems() words, bin_total needs `bins` words.
template <class P>
inline void run_partition_pass(const P& pol, int n_host, const int* d_n, int bins, int nbits, const ChunkPlan& plan,
                               uint32_t* H, uint32_t* bin_total, int32_t* totals_out, int32_t* offsets_out,
                               hipStream_t stream, const char* tag_hist, const char* tag_scan, const char* tag_scatter) {
    NP_LAUNCH(tag_hist, part_hist_kernel<P>, dim3(plan.num_chunks), dim3(kHistThreads), sizeof(uint32_t) * bins, stream,
              pol, n_host, d_n, bins, plan, H);
    NP_LAUNCH(tag_scan, part_colscan_kernel<kColscanThreads>, dim3((bins + kWave - 1) / kWave), dim3(kColscanThreads), 0, stream, H,
              plan.num_chunks, bins, bin_total);
    const size_t lds = part_scatter_lds_bytes<typename P::KeyT>(bins, P::kStageDigit);
    const bool aliased = part_stage_aliased<typename P::KeyT>(bins, P::kStageDigit);
    const void* fn = aliased ? reinterpret_cast<const void*>(part_scatter_kernel<P, true>)
                             : reinterpret_cast<const void*>(part_scatter_kernel<P, false>);
    if (lds > 48 * 1024) {
        // above the default dynamic-LDS allowance: opt in, once per device, kernel and size (a failure shows up as a failed
        // launch); later calls, e.g. while a caller records a graph, then enqueue kernels only
        static std::atomic<int> granted[2][kMaxDevices];
        int dev = 0;
        (void)hipGetDevice(&dev);
        const bool tracked = dev >= 0 && dev < kMaxDevices;
        if (!tracked || granted[aliased][dev].load(std::memory_order_relaxed) < static_cast<int>(lds)) {
            (void)hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (tracked) granted[aliased][dev].store(static_cast<int>(lds), std::memory_order_relaxed);
        }
    }
    if (aliased)
        NP_LAUNCH(tag_scatter, (part_scatter_kernel<P, true>), dim3(plan.num_chunks), dim3(kPartThreads), lds, stream, pol, n_host,
                  d_n, bins, nbits, plan, H, bin_total, totals_out, offsets_out);
    else
        NP_LAUNCH(tag_scatter, (part_scatter_kernel<P, false>), dim3(plan.num_chunks), dim3(kPartThreads), lds, stream, pol, n_host,
                  d_n, bins, nbits, plan, H, bin_total, totals_out, offsets_out);
}

}  // namespace np
