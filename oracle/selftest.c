/*
 * Stand-alone self-check of the CPU oracle (test infrastructure), meant to be built with the address and
 * undefined-behaviour sanitizers:
 *     gcc -std=c11 -g -fsanitize=address,undefined -static-libasan oracle/np_oracle.c oracle/selftest.c -lm
 * It runs the oracle on small pseudo-random inputs and checks four properties that any correct
 * implementation of the path has:
 *   1. the inverse indices reconstruct the input keys;
 *   2. the per-shard splits sum to the number of distinct keys, and every key sits in its owner's segment;
 *   3. pooled outputs equal a brute-force loop;
 *   4. two consecutive batches with overlapping keys, run as lookup -> update -> lookup, give the sequential
 *      result, and rows outside the first batch keep their bits (Eq. (2)).
 * Exit status 0 on success, the number of the failed check otherwise.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int np_ref_dedup(const int64_t*, int32_t, int64_t*, int32_t*, int32_t*, int32_t*, int32_t*, int32_t*);
int32_t np_ref_shard(int64_t, int32_t, int32_t);
int np_ref_route(const int64_t*, int32_t, int32_t, int32_t, int64_t*, int32_t*, int32_t*, int32_t*, int32_t*);
int np_ref_compose(const int32_t*, int32_t, const int32_t*, int32_t*);
int np_ref_lookup_fwd(const float*, int64_t, int32_t, const int64_t*, int32_t, const int32_t*, const int32_t*, int32_t, int32_t,
                      int32_t, int32_t, int32_t, void*, float*, double*);
int np_ref_lookup_bwd(const void*, int32_t, int32_t, int32_t, int32_t, const int32_t*, int32_t, int32_t, const int32_t*, int32_t,
                      const int32_t*, float*, double*);
int np_ref_sparse_adagrad(float*, float*, int64_t, int32_t, const int64_t*, const float*, int32_t, float, float);

static uint64_t rng_state = 88172645463325252ull;
static uint32_t rnd(void) {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 16);
}

enum { R = 300, D = 8, B = 50, MAXL = 6, S = 7 };

typedef struct {
    int32_t n;
    int64_t keys[B * MAXL];
    int32_t off[B + 1];
    float dY[B * D];
} batch_t;

static void make_batch(batch_t* b) {
    b->n = 0;
    b->off[0] = 0;
    for (int i = 0; i < B; ++i) {
        int len = (int)(rnd() % (MAXL + 1));
        for (int k = 0; k < len; ++k) b->keys[b->n++] = (int64_t)((rnd() % 17 == 0) ? 5 : rnd() % R);
        b->off[i + 1] = b->n;
    }
    for (int i = 0; i < B * D; ++i) b->dY[i] = (float)((int)(rnd() % 2001) - 1000) / 500.0f;
}

int main(void) {
    static float table[R * D], state[R], table0[R * D];
    for (int i = 0; i < R * D; ++i) table[i] = (float)((int)(rnd() % 2001) - 1000) / 1e5f;
    memset(state, 0, sizeof(state));
    batch_t b1, b2;
    make_batch(&b1);
    make_batch(&b2);
    static int64_t unique[B * MAXL], send_keys[B * MAXL];
    static int32_t inverse[B * MAXL], counts[B * MAXL], occ_off[B * MAXL + 1], occ[B * MAXL], splits[S], send_off[S + 1],
        sfu[B * MAXL], uts[B * MAXL], l2s[B * MAXL];
    static float out[B * D], out2[B * D], grads[B * MAXL * D];
    int32_t U = -1;
    batch_t* bs[2] = {&b1, &b2};
    for (int t = 0; t < 2; ++t) {
        batch_t* b = bs[t];
        memcpy(table0, table, sizeof(table));
        if (np_ref_dedup(b->keys, b->n, unique, inverse, counts, occ_off, occ, &U)) return 10;
        for (int j = 0; j < b->n; ++j)
            if (unique[inverse[j]] != b->keys[j]) return 1;
        if (np_ref_route(unique, U, S, 1, send_keys, splits, send_off, sfu, uts)) return 11;
        int32_t tot = 0;
        for (int s = 0; s < S; ++s) tot += splits[s];
        if (tot != U) return 2;
        for (int s = 0; s < S; ++s)
            for (int p = send_off[s]; p < send_off[s + 1]; ++p)
                if (np_ref_shard(send_keys[p], S, 1) != s) return 2;
        if (np_ref_compose(inverse, b->n, uts, l2s)) return 12;
        if (np_ref_lookup_fwd(table, R, D, send_keys, U, l2s, b->off, B, b->n, 0, 1, 0, out, NULL, NULL)) return 13;
        for (int i = 0; i < B; ++i)
            for (int d = 0; d < D; ++d) {
                double acc = 0.0;
                for (int j = b->off[i]; j < b->off[i + 1]; ++j) acc += (double)table[b->keys[j] * D + d];
                if (out[i * D + d] != (float)acc) return 3;
            }
        if (np_ref_lookup_bwd(b->dY, 0, D, 0, 1, b->off, B, b->n, inverse, U, uts, grads, NULL)) return 14;
        if (np_ref_sparse_adagrad(table, state, R, D, send_keys, grads, U, 0.01f, 1e-8f)) return 15;
        /* rows outside the batch keep their bits */
        for (int r = 0; r < R; ++r) {
            int touched = 0;
            for (int u = 0; u < U; ++u) touched |= unique[u] == r;
            if (!touched && memcmp(table + r * D, table0 + r * D, sizeof(float) * D)) return 4;
        }
        if (t == 0) {
            /* the second lookup must see the update: forward of batch 2 from the updated table differs from a
               forward from the stale copy exactly when the batches share a key that moved */
            int32_t U2;
            static int64_t u2[B * MAXL];
            static int32_t inv2[B * MAXL], c2[B * MAXL], oo2[B * MAXL + 1], o2[B * MAXL];
            if (np_ref_dedup(b2.keys, b2.n, u2, inv2, c2, oo2, o2, &U2)) return 16;
            np_ref_lookup_fwd(table, R, D, u2, U2, inv2, b2.off, B, b2.n, 0, 1, 0, out, NULL, NULL);
            np_ref_lookup_fwd(table0, R, D, u2, U2, inv2, b2.off, B, b2.n, 0, 1, 0, out2, NULL, NULL);
            int shared_moved = 0;
            for (int a = 0; a < U; ++a)
                for (int c = 0; c < U2; ++c)
                    if (unique[a] == u2[c] && memcmp(table + unique[a] * D, table0 + unique[a] * D, sizeof(float) * D)) shared_moved = 1;
            if (shared_moved != (memcmp(out, out2, sizeof(out)) != 0)) return 4;
        }
    }
    printf("oracle selftest ok\n");
    return 0;
}
