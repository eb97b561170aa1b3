/*
 * CPU oracle for one worker's sparse embedding path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain statement of what each step computes.  It is used by the
 * tests, by the smoke check and by the benchmark's CPU-baseline leg, and by nothing else:
 * the product (the HIP library) never links, loads or calls it, and it shares no code,
 * header, table or helper with the HIP sources.
 *
 * The paper names the operations of the path (Section IV-A: keys are deduplicated, bucketed
 * by the table-sharding rule, the owner queries the vectors of the deduplicated keys, the
 * requester runs forward/backward on the complete set of vectors of its batch, gradients
 * are aggregated at the owner and applied to the vectors in place; Section VI, Eq. (1)-(2):
 * a key outside K(B_t) keeps its vector, a key inside moves by the aggregated gradient) but
 * gives no algorithm for them, so every function below is the textbook definition of the
 * operation written as loops.  Floating point accumulates in fp64 and is rounded once to
 * the storage type.  Nothing is blocked, fused or reordered.
 *
 * Conventions that the paper leaves open and that are fixed here (each is pinned by a test
 * on the CPU against a library routine, a closed form or brute force):
 *   - unique keys come out in ascending order; occurrence lists are stable;
 *   - buckets keep the ascending order of the unique keys (stable bucketing);
 *   - the routing hash is np_ref_mix below (a convention, not a result);
 *   - the optimizer is row-wise Adagrad with the MEAN of squared gradients over the row
 *     and eps outside the square root (the paper's Eq. (2) is plain SGD; the benchmark
 *     definition asks for row-wise Adagrad);
 *   - an empty bag pools to zeros and sends no gradient;
 *   - sequence output is bf16 (round to nearest even), zero padded to max_len;
 *   - a table kept in bf16 or fp16 is read exactly (every such value is an fp32 value) and an updated row is the
 *     fp64 result rounded once to that format, nearest, ties to even (no stochastic rounding, no fp32 shadow copy).
 *
 * All functions return 0 on success, a negative value on a bad argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REF_POOL_SUM 0
#define REF_POOL_MEAN 1
#define REF_SEQ 2
#define REF_F32 0
#define REF_BF16 1
#define REF_F16 2
#define REF_SHARD_MOD 0
#define REF_SHARD_HASH 1

/* ---------------------------------------------------------------- bf16 <-> fp32 ---- */

/* Round an fp32 value to bf16, nearest, ties to even.  NaN stays NaN (quiet bit set). */
uint16_t np_ref_f32_to_bf16(float x) {
    uint32_t b;
    memcpy(&b, &x, 4);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x0040u);
    uint32_t lsb = (b >> 16) & 1u;
    b += 0x7FFFu + lsb;
    return (uint16_t)(b >> 16);
}

float np_ref_bf16_to_f32(uint16_t h) {
    uint32_t b = ((uint32_t)h) << 16;
    float x;
    memcpy(&x, &b, 4);
    return x;
}

/*
 * Round an fp64 value to a binary format with `sig` significant bits whose subnormals are multiples of 2^qmin, in
 * one step, nearest, ties to even (going through fp32 first would round twice).  The result is returned as the fp64
 * value of the rounded number (exact); the caller encodes it.  x is finite and non-zero.
 */
static double ref_round_sig(double a, int sig, int qmin) {
    int e;
    (void)frexp(a, &e);            /* a = m * 2^e with m in [0.5, 1) */
    int q = e - sig;               /* keep `sig` significant bits: the result is an integer times 2^q */
    if (q < qmin) q = qmin;        /* subnormal range: fixed spacing */
    return ldexp(rint(ldexp(a, -q)), q); /* rint: the default rounding mode is nearest-even; both scalings are exact */
}

/* bf16: 8 significant bits, exponents like fp32, subnormals that are multiples of 2^-133. */
uint16_t np_ref_f64_to_bf16(double x) {
    if (isnan(x)) return 0x7FC0u;
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
    double r = ref_round_sig(a, 8, -133);
    if (r >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80u);
    float f = (float)r;            /* exact: r has at most 8 significant bits in fp32's range */
    uint32_t b;
    memcpy(&b, &f, 4);
    return (uint16_t)(sign | (uint16_t)(b >> 16));
}

/* IEEE binary16: 11 significant bits, 5 exponent bits (bias 15), subnormals that are multiples of 2^-24. */
uint16_t np_ref_f64_to_f16(double x) {
    if (isnan(x)) return 0x7E00u;
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7C00u);
    double r = ref_round_sig(a, 11, -24);
    if (r >= 65536.0) return (uint16_t)(sign | 0x7C00u);   /* above the largest finite value 65504 after rounding */
    if (r == 0.0) return sign;
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)ldexp(r, 24));   /* subnormal: the integer r / 2^-24 */
    int e;
    double m = frexp(r, &e);       /* r = m * 2^e, m in [0.5, 1): value 1.f * 2^(e-1) */
    uint16_t frac = (uint16_t)(ldexp(m, 11) - 1024.0);     /* the 10 fraction bits */
    return (uint16_t)(sign | (uint16_t)((e - 1 + 15) << 10) | frac);
}

float np_ref_f16_to_f32(uint16_t h) {
    int e = (h >> 10) & 0x1F, f = h & 0x3FF;
    double v;
    if (e == 0) v = ldexp((double)f, -24);
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return (float)((h & 0x8000u) ? -v : v);
}

/* ---------------------------------------------------------------- step 1: dedup ---- */

typedef struct {
    int64_t key;
    int32_t pos;
} ref_pair;

static int ref_pair_cmp(const void* a, const void* b) {
    const ref_pair* x = (const ref_pair*)a;
    const ref_pair* y = (const ref_pair*)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

/*
 * Section IV-A, "Key Routing": the keys of the batch are deduplicated first.
 * unique       = the distinct keys, ascending
 * inverse[j]   = index in unique of keys[j]
 * counts[u]    = how many j have keys[j] == unique[u]
 * occ          = positions 0..n-1 ordered by (key, position): the stable argsort of keys
 * occ_offsets  = exclusive prefix sum of counts, occ_offsets[U] = n
 * Buffers unique, counts need room for n entries, occ_offsets for n+1.
 */
int np_ref_dedup(const int64_t* keys, int32_t n, int64_t* unique, int32_t* inverse, int32_t* counts,
                 int32_t* occ_offsets, int32_t* occ, int32_t* num_unique) {
    if (n < 0 || !num_unique || !occ_offsets) return -1;
    if (n == 0) {
        *num_unique = 0;
        occ_offsets[0] = 0;
        return 0;
    }
    if (!keys || !unique || !inverse || !counts || !occ) return -1;
    ref_pair* p = (ref_pair*)malloc(sizeof(ref_pair) * (size_t)n);
    if (!p) return -2;
    for (int32_t j = 0; j < n; ++j) {
        p[j].key = keys[j];
        p[j].pos = j;
    }
    qsort(p, (size_t)n, sizeof(ref_pair), ref_pair_cmp);
    int32_t U = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (i == 0 || p[i].key != p[i - 1].key) {
            unique[U] = p[i].key;
            counts[U] = 0;
            occ_offsets[U] = i;
            ++U;
        }
        counts[U - 1] += 1;
        occ[i] = p[i].pos;
        inverse[p[i].pos] = U - 1;
    }
    occ_offsets[U] = n;
    *num_unique = U;
    free(p);
    return 0;
}

/* ---------------------------------------------------------------- step 2: route ---- */

/* The routing hash: a bijection of 64-bit words (odd multiplier, xor-shift, twice). */
uint64_t np_ref_mix(uint64_t k) {
    const uint64_t C = 0x9E3779B97F4A7C15ull;
    uint64_t a = k * C;
    a ^= a >> 32;
    a *= C;
    a ^= a >> 29;
    return a;
}

/* Owner shard of a key under the table-sharding rule (Section IV-A). */
int32_t np_ref_shard(int64_t key, int32_t num_shards, int32_t shard_fn) {
    uint64_t k = (uint64_t)key;
    if (shard_fn == REF_SHARD_HASH) k = np_ref_mix(k);
    return (int32_t)(k % (uint64_t)num_shards);
}

/*
 * Section IV-A, "Key Routing": deduplicated keys are partitioned into one bucket per owner;
 * the buckets, laid end to end, are what the key All2All sends.
 * splits[s]           = number of unique keys owned by shard s
 * send_offsets        = exclusive prefix sum of splits, send_offsets[S] = U
 * send_from_unique[p] = index in unique of the key in send slot p (stable: ascending inside a bucket)
 * send_keys[p]        = unique[send_from_unique[p]]
 * unique_to_send      = the inverse permutation
 */
int np_ref_route(const int64_t* unique, int32_t U, int32_t num_shards, int32_t shard_fn, int64_t* send_keys,
                 int32_t* splits, int32_t* send_offsets, int32_t* send_from_unique, int32_t* unique_to_send) {
    if (U < 0 || num_shards < 1 || !splits || !send_offsets) return -1;
    if (shard_fn != REF_SHARD_MOD && shard_fn != REF_SHARD_HASH) return -1;
    for (int32_t s = 0; s < num_shards; ++s) splits[s] = 0;
    for (int32_t u = 0; u < U; ++u) splits[np_ref_shard(unique[u], num_shards, shard_fn)] += 1;
    send_offsets[0] = 0;
    for (int32_t s = 0; s < num_shards; ++s) send_offsets[s + 1] = send_offsets[s] + splits[s];
    int32_t* cursor = (int32_t*)malloc(sizeof(int32_t) * (size_t)num_shards);
    if (!cursor) return -2;
    for (int32_t s = 0; s < num_shards; ++s) cursor[s] = send_offsets[s];
    for (int32_t u = 0; u < U; ++u) {
        int32_t s = np_ref_shard(unique[u], num_shards, shard_fn);
        int32_t p = cursor[s]++;
        send_keys[p] = unique[u];
        send_from_unique[p] = u;
        unique_to_send[u] = p;
    }
    free(cursor);
    return 0;
}

/* lookup_to_send[j] = unique_to_send[inverse[j]]: the send slot whose vector lookup j reads. */
int np_ref_compose(const int32_t* inverse, int32_t n, const int32_t* unique_to_send, int32_t* lookup_to_send) {
    if (n < 0) return -1;
    for (int32_t j = 0; j < n; ++j) lookup_to_send[j] = unique_to_send[inverse[j]];
    return 0;
}

/* ---------------------------------------------------------------- step 3: forward -- */

/*
 * Section IV-A, "Embedding Retrieval" and the start of "Fwd/Bwd": the vectors of the key list
 * are read from the table and each lookup j of the batch receives the vector of its key,
 *     value_j = table[list_keys[idx[j]], :]        (idx == NULL: list_keys has n entries, idx[j] = j).
 * SUM : out[b,:] = sum of value_j over the lookups of bag b
 * MEAN: that sum divided by the bag length (an empty bag gives zeros)
 * SEQ : out[b,p,:] = value of the p-th lookup of bag b, zeros for p >= length, up to max_len
 * out is fp32 or bf16 (rounded once from the fp64 result).
 * rows_out (optional) [num_list, dim] = table[list_keys[p], :], a bit copy.
 * abs_out (optional, same shape as out, fp64) = sum of |value_j| per element, the scale
 * that a tolerance on a floating-point sum is measured against.
 */
int np_ref_lookup_fwd(const float* table, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                      int32_t num_list, const int32_t* idx, const int32_t* bag_offsets, int32_t num_bags,
                      int32_t n, int32_t mode, int32_t max_len, int32_t out_dtype, void* out, float* rows_out,
                      double* abs_out) {
    if (!table || dim < 1 || num_bags < 0 || n < 0 || num_list < 0) return -1;
    if (mode == REF_SEQ && max_len < 1) return -1;
    double* acc = (double*)malloc(sizeof(double) * (size_t)dim);
    double* aab = (double*)malloc(sizeof(double) * (size_t)dim);
    if (!acc || !aab) { free(acc); free(aab); return -2; }
    size_t per_bag = (mode == REF_SEQ) ? (size_t)max_len * (size_t)dim : (size_t)dim;
    for (int32_t b = 0; b < num_bags; ++b) {
        int32_t lo = bag_offsets[b], hi = bag_offsets[b + 1];
        int32_t len = hi - lo;
        if (mode == REF_SEQ) {
            if (len > max_len) { free(acc); free(aab); return -3; }
            for (int32_t p = 0; p < max_len; ++p) {
                for (int32_t d = 0; d < dim; ++d) {
                    double v = 0.0;
                    if (p < len) {
                        int32_t j = lo + p;
                        int32_t slot = idx ? idx[j] : j;
                        if (slot < 0 || slot >= num_list) { free(acc); free(aab); return -3; }
                        int64_t row = list_keys[slot];
                        if (row < 0 || row >= num_rows) { free(acc); free(aab); return -3; }
                        v = (double)table[(size_t)row * (size_t)dim + (size_t)d];
                    }
                    size_t o = (size_t)b * per_bag + (size_t)p * (size_t)dim + (size_t)d;
                    if (out_dtype == REF_BF16)
                        ((uint16_t*)out)[o] = np_ref_f32_to_bf16((float)v);
                    else
                        ((float*)out)[o] = (float)v;
                    if (abs_out) abs_out[o] = fabs(v);
                }
            }
            continue;
        }
        for (int32_t d = 0; d < dim; ++d) acc[d] = aab[d] = 0.0;
        for (int32_t j = lo; j < hi; ++j) {
            int32_t slot = idx ? idx[j] : j;
            if (slot < 0 || slot >= num_list) { free(acc); free(aab); return -3; }
            int64_t row = list_keys[slot];
            if (row < 0 || row >= num_rows) { free(acc); free(aab); return -3; }
            for (int32_t d = 0; d < dim; ++d) {
                double v = (double)table[(size_t)row * (size_t)dim + (size_t)d];
                acc[d] += v;
                aab[d] += fabs(v);
            }
        }
        for (int32_t d = 0; d < dim; ++d) {
            double v = acc[d], a = aab[d];
            if (mode == REF_POOL_MEAN && len > 0) {
                v /= (double)len;
                a /= (double)len;
            }
            size_t o = (size_t)b * per_bag + (size_t)d;
            if (out_dtype == REF_BF16)
                ((uint16_t*)out)[o] = np_ref_f32_to_bf16((float)v);
            else
                ((float*)out)[o] = (float)v;
            if (abs_out) abs_out[o] = a;
        }
    }
    if (rows_out) {
        for (int32_t p = 0; p < num_list; ++p) {
            int64_t row = list_keys[p];
            if (row < 0 || row >= num_rows) { free(acc); free(aab); return -3; }
            memcpy(rows_out + (size_t)p * (size_t)dim, table + (size_t)row * (size_t)dim, sizeof(float) * (size_t)dim);
        }
    }
    free(acc);
    free(aab);
    return 0;
}

/* ---------------------------------------------------------------- step 4: backward - */

/*
 * Section II-A / IV-A: the gradients of the embeddings are aggregated per key (Eq. (2) sums
 * the per-sample gradients of e_k over the batch).  With the pooling of step 3,
 *     g[u,:] = sum over lookups j with inverse[j] == u of  w_j * dY_j
 *     SUM : dY_j = dY[bag(j),:],                 w_j = 1
 *     MEAN: dY_j = dY[bag(j),:],                 w_j = 1 / length(bag(j))
 *     SEQ : dY_j = dY[bag(j), j - start(bag(j)),:], w_j = 1     (padding positions are never read)
 * dY is fp32 or bf16.  The row of key u is stored at grads[unique_to_send[u],:]
 * (unique_to_send == NULL: at grads[u,:]).  abs_out (optional, [U,dim] fp64, same placement)
 * receives sum |w_j * dY_j|.
 */
int np_ref_lookup_bwd(const void* dY, int32_t dy_dtype, int32_t dim, int32_t mode, int32_t max_len,
                      const int32_t* bag_offsets, int32_t num_bags, int32_t n, const int32_t* inverse,
                      int32_t num_unique, const int32_t* unique_to_send, float* grads, double* abs_out) {
    if (dim < 1 || num_bags < 0 || n < 0 || num_unique < 0) return -1;
    if (mode == REF_SEQ && max_len < 1) return -1;
    size_t total = (size_t)num_unique * (size_t)dim;
    double* acc = (double*)calloc(total ? total : 1, sizeof(double));
    if (!acc) return -2;
    if (abs_out)
        for (size_t i = 0; i < total; ++i) abs_out[i] = 0.0;
    for (int32_t b = 0; b < num_bags; ++b) {
        int32_t lo = bag_offsets[b], hi = bag_offsets[b + 1];
        int32_t len = hi - lo;
        double w = (mode == REF_POOL_MEAN && len > 0) ? 1.0 / (double)len : 1.0;
        for (int32_t j = lo; j < hi; ++j) {
            int32_t u = inverse[j];
            if (u < 0 || u >= num_unique) { free(acc); return -3; }
            size_t dst = (size_t)(unique_to_send ? unique_to_send[u] : u) * (size_t)dim;
            size_t src = (mode == REF_SEQ) ? ((size_t)b * (size_t)max_len + (size_t)(j - lo)) * (size_t)dim
                                           : (size_t)b * (size_t)dim;
            for (int32_t d = 0; d < dim; ++d) {
                double y = (dy_dtype == REF_BF16) ? (double)np_ref_bf16_to_f32(((const uint16_t*)dY)[src + d])
                                                  : (double)((const float*)dY)[src + d];
                acc[dst + d] += w * y;
                if (abs_out) abs_out[dst + d] += fabs(w * y);
            }
        }
    }
    for (size_t i = 0; i < total; ++i) grads[i] = (float)acc[i];
    free(acc);
    return 0;
}

/* ---------------------------------------------------------------- step 5: update --- */

/*
 * Section IV-B: the gradients are applied directly to the vectors in the active buffer;
 * Eq. (2): only keys of the batch move.  Row-wise Adagrad, for each list slot p with key k
 * and gradient row g = grads[p,:]:
 *     G        = state[k] + (1/dim) * sum_d g_d^2
 *     state[k] = G
 *     table[k,d] = table[k,d] - lr * g_d / (sqrt(G) + eps)
 * Keys in the list are pairwise distinct.  Every other row and state entry is untouched.
 */
int np_ref_sparse_adagrad(float* table, float* state, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                          const float* grads, int32_t num_list, float lr, float eps) {
    if (!table || !state || dim < 1 || num_list < 0) return -1;
    for (int32_t p = 0; p < num_list; ++p) {
        int64_t k = list_keys[p];
        if (k < 0 || k >= num_rows) return -3;
        const float* g = grads + (size_t)p * (size_t)dim;
        double ss = 0.0;
        for (int32_t d = 0; d < dim; ++d) ss += (double)g[d] * (double)g[d];
        double G = (double)state[k] + ss / (double)dim;
        state[k] = (float)G;
        double denom = sqrt(G) + (double)eps;
        float* w = table + (size_t)k * (size_t)dim;
        for (int32_t d = 0; d < dim; ++d) w[d] = (float)((double)w[d] - (double)lr * (double)g[d] / denom);
    }
    return 0;
}

/*
 * The same update on a table stored in 16 bits (bit patterns, [num_rows, dim]; table_dtype REF_BF16 or REF_F16); the
 * state stays fp32.  The old row is widened exactly, the step is taken in fp64 with the fp64 state sum, and the new
 * row is rounded once to the storage format.
 */
int np_ref_sparse_adagrad_16(uint16_t* table, int32_t table_dtype, float* state, int64_t num_rows, int32_t dim,
                             const int64_t* list_keys, const float* grads, int32_t num_list, float lr, float eps) {
    if (!table || !state || dim < 1 || num_list < 0) return -1;
    if (table_dtype != REF_BF16 && table_dtype != REF_F16) return -1;
    for (int32_t p = 0; p < num_list; ++p) {
        int64_t k = list_keys[p];
        if (k < 0 || k >= num_rows) return -3;
        const float* g = grads + (size_t)p * (size_t)dim;
        double ss = 0.0;
        for (int32_t d = 0; d < dim; ++d) ss += (double)g[d] * (double)g[d];
        double G = (double)state[k] + ss / (double)dim;
        state[k] = (float)G;
        double denom = sqrt(G) + (double)eps;
        uint16_t* w = table + (size_t)k * (size_t)dim;
        for (int32_t d = 0; d < dim; ++d) {
            double old = table_dtype == REF_BF16 ? (double)np_ref_bf16_to_f32(w[d]) : (double)np_ref_f16_to_f32(w[d]);
            double upd = old - (double)lr * (double)g[d] / denom;
            w[d] = table_dtype == REF_BF16 ? np_ref_f64_to_bf16(upd) : np_ref_f64_to_f16(upd);
        }
    }
    return 0;
}

int np_ref_sparse_adagrad_bf16(uint16_t* table, float* state, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                               const float* grads, int32_t num_list, float lr, float eps) {
    return np_ref_sparse_adagrad_16(table, REF_BF16, state, num_rows, dim, list_keys, grads, num_list, lr, eps);
}

/* ------------------------------------------------- dual-buffer synchronisation (Section IV-B) -------- */

/*
 * Section IV-B: before batch B_t starts its forward pass, the intersection of the compact key sets of the two
 * consecutive batches is taken (on keys, not on vectors).  keys_a and keys_b are ascending and distinct.
 * Output, in ascending key order: pairs (idx_a[i], idx_b[i]) with keys_a[idx_a[i]] == keys_b[idx_b[i]].
 * A plain two-pointer merge.
 */
int np_ref_intersect(const int64_t* keys_a, int32_t na, const int64_t* keys_b, int32_t nb, int32_t* idx_a,
                     int32_t* idx_b, int32_t* num_common) {
    if (na < 0 || nb < 0 || !num_common) return -1;
    int32_t i = 0, j = 0, c = 0;
    while (i < na && j < nb) {
        if (keys_a[i] < keys_b[j]) {
            ++i;
        } else if (keys_b[j] < keys_a[i]) {
            ++j;
        } else {
            idx_a[c] = i;
            idx_b[c] = j;
            ++c;
            ++i;
            ++j;
        }
    }
    *num_common = c;
    return 0;
}

/*
 * Section IV-B: the vectors of the intersecting keys are copied from the active buffer (which holds the
 * updates of B_{t-1}) into the prefetch buffer (which was filled for B_t before those updates): Eq. (2),
 * second case.  dst[dst_idx[i], :] = src[src_idx[i], :] for i < count, a bit copy.
 */
int np_ref_sync_rows(const float* src, const int32_t* src_idx, float* dst, const int32_t* dst_idx, int32_t count,
                     int32_t dim) {
    if (count < 0 || dim < 1) return -1;
    for (int32_t i = 0; i < count; ++i)
        memcpy(dst + (size_t)dst_idx[i] * (size_t)dim, src + (size_t)src_idx[i] * (size_t)dim, sizeof(float) * (size_t)dim);
    return 0;
}
