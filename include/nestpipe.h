/*
 * nestpipe.h - C ABI of the MI355X (gfx950) sparse-embedding hot path.
 *
 * One worker's share of the embedding work that the paper's nested pipelines exist to hide
 * (Section IV-A, stages "Key Routing", "Embedding Retrieval" and "Fwd/Bwd"; Section IV-B for
 * the in-place update; Section VI, Eq. (1)-(2) for what an update must and must not touch):
 *
 *     np_dedup -> np_route -> [key All2All] -> np_lookup_fwd -> [embedding All2All, dense model]
 *              -> np_lookup_bwd -> [gradient All2All] -> np_sparse_adagrad
 *
 * The bracketed exchanges are not part of this library: an All2All is represented by the packed
 * send buffer and the per-shard split counts that np_route produces.
 *
 * General rules
 *  - Every pointer is DEVICE memory owned by the caller unless a comment says "host".  The
 *    library never allocates, frees or keeps a pointer after the call returns.  Scratch memory
 *    is the caller's `ws` buffer, sized by the matching np_*_workspace_bytes() (a pure host
 *    function).  `ws` must be 256-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *    work: they never synchronise with the host.  The number of distinct keys U is data
 *    dependent and lives in device memory (`d_num_unique` / `d_num_list`); the host passes an
 *    upper bound `cap` that sizes buffers and grids.
 *  - Return value: NP_OK or a negative np_status.  Arguments are validated on the host before
 *    anything is enqueued, so a call that returns NP_ERR_INVALID_ARG, NP_ERR_WORKSPACE or
 *    NP_ERR_UNSUPPORTED has written nothing.  Nothing throws, aborts or prints.
 *  - Keys are int64 row ids of one fused table, 0 <= key < num_rows (the caller adds a per-table
 *    base to form them).  Every index, offset and count is int32; a batch holds at most
 *    2^31 - 1 - 2^20 lookups (larger n: NP_ERR_UNSUPPORTED).
 *  - Bags: the lookups of bag b are keys[bag_offsets[b] .. bag_offsets[b+1]), bag_offsets is
 *    non-decreasing with bag_offsets[0] = 0 and bag_offsets[num_bags] = n.  Empty bags are legal.
 *  - Out-of-range keys, repeated keys in an update list, or offsets that break the rules above
 *    are precondition violations (not checked on the device).
 *  - Supported row widths: dim a multiple of 4, 4 <= dim <= 1024; table, gradient and output
 *    buffers 16-byte aligned (8-byte for 16-bit tables, bf16 outputs and bf16 dY; a bf16 dY at a
 *    16-byte aligned address is read with wider loads, with the same result).
 *  - The compute calls keep no state between calls and act on the calling thread's current
 *    device: they may be issued from several host threads and on several devices.  Ordering
 *    calls that share a buffer (through streams and events) is the caller's job.  The np_prof_*
 *    timing hooks are the exception (process-wide state, one thread at a time).
 *  - The first np_dedup / np_route / np_lookup_bwd call of a process on a device opts its partition kernel in to
 *    more than 48 KB of dynamic LDS (hipFuncSetAttribute, once per device; no stream work, no allocation).
 *    Record a HIP graph after one ordinary call has been made.
 */
#ifndef NESTPIPE_H_
#define NESTPIPE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum np_status {
    NP_OK = 0,
    NP_ERR_INVALID_ARG = -1, /* null required pointer, negative size, bad enum value, misaligned buffer */
    NP_ERR_WORKSPACE = -2,   /* ws is NULL/misaligned or ws_bytes is below np_*_workspace_bytes() */
    NP_ERR_UNSUPPORTED = -3, /* legal request outside what the kernels cover (dim, num_shards, sizes) */
    NP_ERR_HIP = -4          /* a launch failed; the HIP error was consumed with hipGetLastError */
} np_status;

enum { NP_SHARD_MOD = 0, NP_SHARD_HASH = 1 };
enum { NP_POOL_SUM = 0, NP_POOL_MEAN = 1, NP_SEQ = 2 };
enum { NP_F32 = 0, NP_BF16 = 1, NP_F16 = 2 };  /* NP_F16 (IEEE binary16) is a table dtype only */

#define NP_MAX_SHARDS 4096
#define NP_ROUTE_STATIC_MAX_SHARDS 2048 /* np_route_static: shards its built-in scratch is sized for */
#define NP_MAX_DIM 1024

/* Library version (major * 10000 + minor * 100 + patch).  Host function. */
int np_version(void);

/* Static text for a status code.  Host function; the pointer is to a string literal. */
const char* np_status_string(int status);

/*
 * np_dedup - Section IV-A, "Key Routing": the sparse keys of the batch are deduplicated first
 * (and again on the owner over the keys received from all sources, "Embedding Retrieval").
 *
 *   keys         [n]   in   int64, only the low key_bits bits may be non-zero (1 <= key_bits <= 63)
 *   unique       [n]   out  the U distinct keys, ascending; entries >= U are not written
 *   inverse      [n]   out  inverse[j] = index of keys[j] in unique; optional (NULL: not produced, which saves the
 *                           random 4-byte scatter; a worker that reads its own table by key does not need it)
 *   counts       [n]   out  counts[u] = multiplicity of unique[u], u < U
 *   occ_offsets  [n+1] out  exclusive prefix sum of counts; occ_offsets[U] = n
 *   occ          [n]   out  positions 0..n-1 sorted by (key, position): the stable argsort of keys.
 *                           occ[occ_offsets[u] .. occ_offsets[u+1]) are the lookups of unique[u].
 *   d_num_unique [1]   out  U
 *
 * All outputs are bit-exact functions of the input (no dependence on scheduling).
 * n = 0 is legal: writes U = 0 and occ_offsets[0] = 0.
 */
int np_dedup(const int64_t* keys, int32_t n, int32_t key_bits, int64_t* unique, int32_t* inverse, int32_t* counts,
             int32_t* occ_offsets, int32_t* occ, int32_t* d_num_unique, void* ws, size_t ws_bytes, void* stream);
size_t np_dedup_workspace_bytes(int32_t n, int32_t key_bits);

/*
 * np_route - Section IV-A, "Key Routing": the deduplicated keys are partitioned into buckets by the
 * table-sharding rule; the buckets laid end to end are the payload of the key All2All.
 *
 *   unique          [cap]   in   ascending distinct keys, the first U = *d_num_unique are valid
 *   d_num_unique    [1]     in   U (device), U <= cap
 *   num_shards              1 <= S <= NP_MAX_SHARDS
 *   shard_fn                NP_SHARD_MOD: shard = key mod S.
 *                           NP_SHARD_HASH: shard = mix(key) mod S with, on uint64 and C = 0x9E3779B97F4A7C15,
 *                           a = key*C; a ^= a>>32; a *= C; a ^= a>>29; mix = a.
 *   send_keys       [cap]   out  keys grouped by shard 0..S-1, ascending inside a shard (stable bucketing)
 *   splits          [S]     out  keys per shard (the All2All send counts); sums to U
 *   send_offsets    [S+1]   out  exclusive prefix sum of splits
 *   send_from_unique[cap]   out  send_keys[p] = unique[send_from_unique[p]]
 *   unique_to_send  [cap]   out  inverse permutation: send_keys[unique_to_send[u]] = unique[u]
 *   inverse         [n]     in   optional (NULL with lookup_to_send NULL): np_dedup's inverse
 *   lookup_to_send  [n]     out  optional: lookup_to_send[j] = unique_to_send[inverse[j]], the send slot whose
 *                                vector lookup j consumes once the owners have answered
 */
int np_route(const int64_t* unique, const int32_t* d_num_unique, int32_t cap, int32_t num_shards, int32_t shard_fn,
             int64_t* send_keys, int32_t* splits, int32_t* send_offsets, int32_t* send_from_unique,
             int32_t* unique_to_send, const int32_t* inverse, int32_t n, int32_t* lookup_to_send, void* ws,
             size_t ws_bytes, void* stream);
size_t np_route_workspace_bytes(int32_t cap, int32_t num_shards);

/*
 * np_route_static - np_route for callers that cannot allocate or hand over a workspace: code recorded under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus ws / ws_bytes), same
 * kernels and bit-identical outputs; the scratch of the pass (the 512 x num_shards histogram matrix and the
 * per-shard totals) lives in a device array built into the library, 4 MiB + 8 KiB per GPU the library runs on,
 * held until the process ends.  The call allocates and frees nothing; the first call on a device looks the
 * array's address up (hipGetSymbolAddress) and keeps it.
 *
 *   num_shards > NP_ROUTE_STATIC_MAX_SHARDS  ->  NP_ERR_UNSUPPORTED (nothing enqueued); cap is not limited.
 *   The address lookup failing               ->  NP_ERR_HIP.
 *
 * Every call on one GPU uses that GPU's one array: calls that may overlap there (different streams, or host
 * threads enqueueing on different streams) race on it and must be ordered by the caller.  Nothing in the array has
 * to start at zero (each pass writes every word it later reads), so calls in a row need no clearing in between.
 */
int np_route_static(const int64_t* unique, const int32_t* d_num_unique, int32_t cap, int32_t num_shards, int32_t shard_fn,
                    int64_t* send_keys, int32_t* splits, int32_t* send_offsets, int32_t* send_from_unique,
                    int32_t* unique_to_send, const int32_t* inverse, int32_t n, int32_t* lookup_to_send, void* stream);

/*
 * np_lookup_fwd - Section IV-A, "Embedding Retrieval" (the owner reads the vectors of the deduplicated
 * keys from its table shard) and the start of "Fwd/Bwd" (the requester holds the vector of every lookup
 * of its batch).  value_j = table[list_keys[idx[j]], :].
 *
 *   table      [num_rows, dim] in  fp32, row-major, HBM resident
 *   list_keys  [cap]  in   key list (np_route's send_keys, or np_dedup's unique)
 *   d_num_list [1]    in   number of valid list entries; read only when rows_out != NULL (may be NULL otherwise)
 *   idx        [n]    in   lookup -> list slot; NULL means list_keys has n entries and lookup j reads slot j
 *              list_keys may be NULL when idx is given: the slot itself is the row, value_j = table[idx[j], :]
 *              (the requester's side of the embedding All2All: pooling straight from the buffer of received rows,
 *              table = that buffer, idx = np_route's lookup_to_send)
 *   mode / out:
 *     NP_POOL_SUM   out[b,:] = sum of value_j over bag b                  out is [num_bags, dim]
 *     NP_POOL_MEAN  the sum times 1/length; an empty bag gives zeros       out is [num_bags, dim]
 *     NP_SEQ        out[b,p,:] = value of the p-th lookup of bag b, zeros for p >= length
 *                   out is [num_bags, max_len, dim]; every bag length must be <= max_len
 *   out_dtype  NP_F32 or NP_BF16 (round to nearest even from the fp32 result); sums accumulate in fp32 in
 *              ascending lookup order
 *   rows_out   [cap, dim]  out, optional: rows_out[p,:] = table[list_keys[p],:] for p < *d_num_list (a bit
 *              copy: the payload of the embedding All2All)
 */
int np_lookup_fwd(const float* table, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                  const int32_t* d_num_list, int32_t cap, const int32_t* idx, const int32_t* bag_offsets,
                  int32_t num_bags, int32_t n, int32_t mode, int32_t max_len, int32_t out_dtype, void* out,
                  float* rows_out, void* ws, size_t ws_bytes, void* stream);
size_t np_lookup_fwd_workspace_bytes(int32_t num_bags, int32_t n, int32_t dim, int32_t mode);

/*
 * np_lookup_bwd - Section II-A and IV-A: embedding gradients are routed to the owner and aggregated per
 * key; Eq. (2): the update of key k uses the sum over the batch of the gradients of e_k.
 *
 *   g[u,:] = sum over lookups j of key unique[u] of  w_j * dY_j
 *     NP_POOL_SUM   dY_j = dY[bag(j),:]                      w_j = 1
 *     NP_POOL_MEAN  dY_j = dY[bag(j),:]                      w_j = 1/length(bag(j))
 *     NP_SEQ        dY_j = dY[bag(j), j - start(bag(j)), :]  w_j = 1   (dY is [num_bags, max_len, dim];
 *                                                                      padding positions are never read)
 *   dY          in   fp32 or bf16 (dy_dtype)
 *   occ_offsets, occ  in   np_dedup's occurrence lists
 *   d_num_unique[1]   in   U (device), U <= cap
 *   unique_to_send [cap] in  optional: the row of key u is written at grads[unique_to_send[u],:]
 *                            (NULL: at grads[u,:])
 *   grads       [cap, dim] out fp32; rows >= U are not written
 *
 * Deterministic: fp32 accumulation in an order that depends only on occ_offsets (never on scheduling),
 * no floating-point atomics; two runs on the same input give identical bits.
 */
int np_lookup_bwd(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                  const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* occ_offsets,
                  const int32_t* occ, const int32_t* d_num_unique, int32_t cap, const int32_t* unique_to_send,
                  float* grads, void* ws, size_t ws_bytes, void* stream);
size_t np_lookup_bwd_workspace_bytes(int32_t num_bags, int32_t n, int32_t dim, int32_t mode);

/*
 * np_lookup_bwd in two parts, for callers that want the part that does not need dY out of the way early (the dense
 * model runs between the forward and the backward; in that time the index work can already be done):
 *
 *   np_lookup_bwd_prepare   everything that depends on the index arrays alone: bag_offsets, occ_offsets, occ (lookup -> bag
 *                           map, first key segment of every tile, the order in which tiles run, the upstream-gradient row
 *                           of every sorted lookup); written into ws.
 *   np_lookup_bwd_prepared  the reduction itself; ws must be the buffer a np_lookup_bwd_prepare call with the same
 *                           dy_dtype, dim, mode, max_len, bag_offsets, num_bags, n, occ_offsets, occ and d_num_unique has
 *                           completed on (order the two through the stream or an event), untouched in between.
 *
 * np_lookup_bwd_prepare followed by np_lookup_bwd_prepared gives the bits of np_lookup_bwd.  Arguments, errors and the
 * workspace size are those of np_lookup_bwd.
 */
int np_lookup_bwd_prepare(int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len, const int32_t* bag_offsets,
                          int32_t num_bags, int32_t n, const int32_t* occ_offsets, const int32_t* occ, const int32_t* d_num_unique,
                          void* ws, size_t ws_bytes, void* stream);
int np_lookup_bwd_prepared(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                           const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* occ_offsets,
                           const int32_t* occ, const int32_t* d_num_unique, int32_t cap, const int32_t* unique_to_send,
                           float* grads, void* ws, size_t ws_bytes, void* stream);

/*
 * np_sparse_adagrad - Section IV-B: gradients are applied directly to the vectors held in HBM; Eq. (2):
 * keys outside the batch keep their vectors bit for bit.  The paper's update is plain SGD; this build's
 * benchmark definition asks for row-wise Adagrad, one fp32 accumulator per row:
 *
 *   for each list slot p < *d_num_list, k = list_keys[p], g = grads[p,:]:
 *     G = state[k] + (1/dim) * sum_d g_d^2 ;  state[k] = G ;  table[k,d] -= lr * g_d / (sqrt(G) + eps)
 *
 *   table [num_rows, dim] in/out,  state [num_rows] in/out,  list_keys pairwise distinct.
 */
int np_sparse_adagrad(float* table, float* state, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                      const float* grads, const int32_t* d_num_list, int32_t cap, float lr, float eps,
                      void* stream);

/*
 * Tables stored in 16 bits (a storage variant of this build; the paper stores fp32 vectors, Section IV-B).
 * table_dtype is NP_F32, NP_BF16 or NP_F16; with NP_F32 the two calls below are np_lookup_fwd and np_sparse_adagrad.
 *
 * np_lookup_fwd_t: a 16-bit row is widened exactly to fp32, then everything is as in np_lookup_fwd (fp32 sums in
 *   ascending lookup order).  rows_out has the table's dtype and is a bit copy.  table and rows_out need 8-byte
 *   alignment for 16-bit rows (16 for fp32).  out_dtype stays NP_F32 or NP_BF16.
 * np_sparse_adagrad_t: the row is widened, the fp32 step of np_sparse_adagrad is taken, and the new row is rounded
 *   to the table's format, nearest, ties to even (no stochastic rounding, no fp32 shadow copy); the state stays
 *   fp32.  A zero gradient leaves the row's bits as they are.
 * Errors as for the fp32 calls, plus NP_ERR_INVALID_ARG for an unknown table_dtype.
 */
int np_lookup_fwd_t(const void* table, int32_t table_dtype, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                    const int32_t* d_num_list, int32_t cap, const int32_t* idx, const int32_t* bag_offsets,
                    int32_t num_bags, int32_t n, int32_t mode, int32_t max_len, int32_t out_dtype, void* out,
                    void* rows_out, void* ws, size_t ws_bytes, void* stream);
int np_sparse_adagrad_t(void* table, int32_t table_dtype, float* state, int64_t num_rows, int32_t dim,
                        const int64_t* list_keys, const float* grads, const int32_t* d_num_list, int32_t cap, float lr,
                        float eps, void* stream);

/*
 * np_lookup_bwd_adagrad - np_lookup_bwd and np_sparse_adagrad in one pass for a worker that owns the rows it
 * reduces (no gradient All2All in between): every finished gradient row is applied on the spot to
 * table[unique[u], :] with the row-wise Adagrad rule above and is never written to HBM (Section IV-B: gradients
 * are applied directly to the vectors of the active buffer).  Same sums, same order, same update arithmetic as
 * the two separate calls: the table and state come out bit-identical.  Every dim the separate calls take.
 *
 *   unique [cap] in  np_dedup's distinct keys (pairwise distinct, so every row is updated exactly once)
 *   other arguments as in np_lookup_bwd / np_sparse_adagrad; workspace as np_lookup_bwd_workspace_bytes.
 */
int np_lookup_bwd_adagrad(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                          const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* occ_offsets,
                          const int32_t* occ, const int64_t* unique, const int32_t* d_num_unique, int32_t cap, float* table,
                          float* state, int64_t num_rows, float lr, float eps, void* ws, size_t ws_bytes, void* stream);
/* The same for a table of dtype NP_F32, NP_BF16 or NP_F16 (the update rounds as np_sparse_adagrad_t does, so the table
 * and state again match the two separate calls bit for bit). */
int np_lookup_bwd_adagrad_t(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                            const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* occ_offsets,
                            const int32_t* occ, const int64_t* unique, const int32_t* d_num_unique, int32_t cap, void* table,
                            int32_t table_dtype, float* state, int64_t num_rows, float lr, float eps, void* ws,
                            size_t ws_bytes, void* stream);

/* ---- dual-buffer synchronisation (Section IV-B) --------------------------------------------------- */

/*
 * np_intersect - Section IV-B: "a dedicated kernel computes the intersection of compact key sets between
 * consecutive batches, rather than full embedding vectors".
 *
 *   keys_a [cap_a] in  ascending distinct keys of B_{t-1} (np_dedup's unique), *d_num_a valid
 *   keys_b [cap_b] in  ascending distinct keys of B_t, *d_num_b valid
 *   idx_a, idx_b [min(cap_a, cap_b)] out  keys_a[idx_a[i]] == keys_b[idx_b[i]] for i < *d_num_common, in
 *                      ascending key order; every common key appears exactly once
 *   d_num_common [1]   out
 * Bit-exact function of the inputs.  Either list may be empty.
 */
int np_intersect(const int64_t* keys_a, const int32_t* d_num_a, int32_t cap_a, const int64_t* keys_b,
                 const int32_t* d_num_b, int32_t cap_b, int32_t* idx_a, int32_t* idx_b, int32_t* d_num_common, void* ws,
                 size_t ws_bytes, void* stream);
size_t np_intersect_workspace_bytes(int32_t cap_b);

/*
 * np_sync_rows - Section IV-B: the vectors of the common keys are copied from the active buffer to the prefetch
 * buffer with device-to-device copies (Eq. (2), second case: a key of B_{t-1} carries its updated vector).
 *
 *   dst_rows[dst_idx[i], :] = src_rows[src_idx[i], :]  for i < *d_count (device), a bit copy of fp32 rows of
 *   width dim.  dst_idx entries are pairwise distinct; rows of dst that are not named keep their bits.
 */
int np_sync_rows(const float* src_rows, const int32_t* src_idx, float* dst_rows, const int32_t* dst_idx,
                 const int32_t* d_count, int32_t cap, int32_t dim, void* stream);

/* ---- harness utilities (not on the hot path) ------------------------------------------------------ */

/*
 * Fill table[row, col] with the stateless initialiser used by the synthetic workloads:
 *   h = (row*dim + col) + seed*0x2545F4914F6CDD1D; h ^= h>>31; h *= 0xD6E8FEB86659FD93; h ^= h>>27;
 *   h *= 0xA3B195354A39B70D; h ^= h>>33;  value = (float)((int)(h>>40) - 2^23) * (0.01f / 2^23)
 * uniform on [-0.01, 0.01), one rounding, identical on every platform.
 */
int np_util_table_init(float* table, int64_t num_rows, int32_t dim, uint64_t seed, void* stream);
/* The same for a table of dtype NP_F32, NP_BF16 or NP_F16 (the value above rounded to that format, nearest even). */
int np_util_table_init_t(void* table, int32_t table_dtype, int64_t num_rows, int32_t dim, uint64_t seed, void* stream);

/*
 * Count the rows of `table` whose bits differ anywhere from what np_util_table_init(seed) wrote: the number
 * of rows an update has touched.  *d_count (device, uint64) is overwritten.  Used by the tests to show at
 * full table size that rows outside a batch keep their bits.
 */
int np_util_table_count_changed(const float* table, int64_t num_rows, int32_t dim, uint64_t seed,
                                unsigned long long* d_count, void* stream);
int np_util_table_count_changed_t(const void* table, int32_t table_dtype, int64_t num_rows, int32_t dim, uint64_t seed,
                                  unsigned long long* d_count, void* stream);

/*
 * Check the preconditions that the hot-path calls do not check on the device (a debugging aid: one pass over the
 * batch).  d_errors (device, 4 x uint64) is overwritten with counts of
 *   [0] keys outside [0, num_rows)            [1] positions b with bag_offsets[b+1] < bag_offsets[b]
 *   [2] 1 if bag_offsets[0] != 0              [3] 1 if bag_offsets[num_bags] != n
 * All four zero means the batch is well formed.  keys may be NULL (n = 0) and bag_offsets may be NULL (num_bags = 0):
 * the corresponding checks are skipped.
 */
int np_util_check_batch(const int64_t* keys, int32_t n, int64_t num_rows, const int32_t* bag_offsets, int32_t num_bags,
                        unsigned long long* d_errors, void* stream);

/*
 * Tunables: thresholds that decide which of two code paths with IDENTICAL results a call takes; they change speed, never
 * a bit of any output.  Process-wide, host functions, safe to call from any thread; a call reads them when it is
 * enqueued (np_lookup_bwd_prepare and np_lookup_bwd_prepared of one batch must see the same values).
 *
 *   "emit_order_min_n"        np_dedup writes the inverse map in a cache-friendly tile order from this many lookups on
 *                             (initially 4194304; smaller batches take fewer launches instead)
 *   "bwd_order_min_dy_bytes"  np_lookup_bwd runs its tiles locality-ordered when the upstream gradient exceeds this many
 *                             bytes (initially 268435456, the last-level cache of an MI355X)
 *   "bwd_row_index"           1: the index part of np_lookup_bwd also resolves the upstream-gradient row of every sorted
 *                             lookup, laid out block by block (one more launch, 4 to 8 bytes per lookup written and read
 *                             again); the reduction then starts its row loads at once.  0 (initially): the reduction
 *                             resolves the rows itself.  On an MI355X the reduction gets 6 % faster and the extra pass
 *                             costs three times that, so it pays only where the index part runs ahead of time, out of
 *                             the way (np_lookup_bwd_prepare while the dense model computes)
 *   "bwd_singles_by_bag"      1: keys with a single lookup (their gradient row is a copy of one upstream row) are served
 *                             bag by bag by a copy kernel, the reduction skips them (pooled modes, fp32 gradients).
 *                             0 (initially).  Measured slower on an MI355X: the reduction drops from 2.0 to 1.4 ms on
 *                             42 M lookups, the three extra passes take 0.8 ms
 *
 * np_tune_set: NP_OK, or NP_ERR_INVALID_ARG for an unknown name or a value outside the knob's range.  np_tune_get: the value, -1 for an
 * unknown name.
 */
int np_tune_set(const char* name /* host */, int64_t value);
int64_t np_tune_get(const char* name /* host */);

/* Plain device copy of `bytes` (multiple of 16) with 16-byte loads and stores: the bandwidth yardstick. */
int np_util_stream_copy(void* dst, const void* src, size_t bytes, void* stream);

/*
 * The gather yardstick: n random reads of whole 256-byte rows (64 floats) from the first num_rows rows of `src`, with the
 * access pattern of the row kernels (16 lanes x 16 bytes per row, eight rows in flight per lane group), summed in groups
 * of 64 into out [n/64, 64] fp32.  Row i read = hash(i, seed) mod num_rows, so num_rows sets the working set: a few
 * thousand rows stay in L2, half a million in the last-level cache, a whole table means HBM.  n a multiple of 64,
 * num_rows < 2^32; src and out 16-byte aligned.  Timing it (HIP events) gives what a gather can reach on this GPU.
 */
int np_util_gather_rate(const float* src, int64_t num_rows, int64_t n, uint32_t seed, float* out, void* stream);

/*
 * Per-kernel timing with HIP events on the caller's stream.  np_prof_enable(1) makes every kernel launch
 * of the library record a start and stop event (events are created on first use and reused);
 * np_prof_collect synchronises those events and copies up to `max_entries` records, in launch order, into
 * host arrays: names[i] points to a static string, ms[i] is the kernel's duration.  Returns the number of
 * records and clears the log.  np_prof_only("a,b") restricts the timing to launches with these names (host string,
 * copied; NULL or "" lifts the restriction), so that a timed run pays for a few events only.  Host functions; not
 * thread safe; meant for the benchmark only.
 */
int np_prof_enable(int on);
int np_prof_only(const char* names /* host */);
int np_prof_collect(const char** names /* host */, float* ms /* host */, int max_entries);

#ifdef __cplusplus
}
#endif
#endif /* NESTPIPE_H_ */
