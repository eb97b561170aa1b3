/*
 * Stand-alone self-check of the CPU oracle (test infrastructure), meant to be built with the address and
 * undefined-behaviour sanitizers:
 *     gcc -std=c11 -g -fsanitize=address,undefined -static-libasan oracle/np_oracle.c oracle/selftest.c -lm
 * It runs the oracle on small pseudo-random inputs and checks five properties that any correct
 * implementation of the path has:
 *   1. the inverse indices reconstruct the input keys;
 *   2. the per-shard splits sum to the number of distinct keys, and every key sits in its owner's segment;
 *   3. pooled outputs equal a brute-force loop;
 *   4. two consecutive batches with overlapping keys, run as lookup -> update -> lookup, give the sequential
 *      result, and rows outside the first batch keep their bits (Eq. (2)).
 *   5. 16-bit tables: decoding and one-step rounding are inverse to each other on every finite bf16 / fp16
 *      pattern, rounding is monotone, and the 16-bit Adagrad step stays within half a spacing of the fp32 one.
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
int np_ref_sparse_adagrad_16(uint16_t*, int32_t, float*, int64_t, int32_t, const int64_t*, const float*, int32_t, float, float);
uint16_t np_ref_f64_to_bf16(double);
uint16_t np_ref_f64_to_f16(double);
float np_ref_bf16_to_f32(uint16_t);
float np_ref_f16_to_f32(uint16_t);

static int check_16bit(void) {
    /* every finite pattern survives decode -> round; rounding is monotone between neighbouring patterns */
    for (int kind = 1; kind <= 2; ++kind) {
        double prev = -INFINITY;
        for (uint32_t h = 0; h < 0x8000u; ++h) {
            float v = kind == 1 ? np_ref_bf16_to_f32((uint16_t)h) : np_ref_f16_to_f32((uint16_t)h);
            if (isnan(v) || isinf(v)) continue;
            uint16_t back = kind == 1 ? np_ref_f64_to_bf16((double)v) : np_ref_f64_to_f16((double)v);
            if (back != h) return 5;
            uint16_t neg = kind == 1 ? np_ref_f64_to_bf16(-(double)v) : np_ref_f64_to_f16(-(double)v);
            if (neg != (uint16_t)(h | 0x8000u)) return 5;
            if (h > 0 && !((double)v > prev)) return 5;
            if (h > 0) {  /* a value just above / below the midpoint of two neighbours goes to the nearer one */
                double mid = 0.5 * ((double)v + prev);
                uint16_t up = kind == 1 ? np_ref_f64_to_bf16(mid * (1.0 + 1e-12)) : np_ref_f64_to_f16(mid * (1.0 + 1e-12));
                uint16_t dn = kind == 1 ? np_ref_f64_to_bf16(mid * (1.0 - 1e-12)) : np_ref_f64_to_f16(mid * (1.0 - 1e-12));
                if (up != h || dn != (uint16_t)(h - 1)) return 5;
            }
            prev = (double)v;
        }
    }
    /* the 16-bit step against the fp32 step on the same (exactly representable) rows */
    enum { R16 = 40, D16 = 8, L16 = 10 };
    for (int kind = 1; kind <= 2; ++kind) {
        uint16_t t16[R16 * D16];
        float t32[R16 * D16], s16[R16], s32[R16], g[L16 * D16];
        int64_t keys[L16];
        for (int i = 0; i < R16 * D16; ++i) {
            double x = ((double)((i * 2654435761u) >> 8 & 0xFFFF) / 65536.0 - 0.5) * 0.05;
            t16[i] = kind == 1 ? np_ref_f64_to_bf16(x) : np_ref_f64_to_f16(x);
            t32[i] = kind == 1 ? np_ref_bf16_to_f32(t16[i]) : np_ref_f16_to_f32(t16[i]);
        }
        for (int r = 0; r < R16; ++r) s16[r] = s32[r] = (float)(r % 3) * 0.01f;
        for (int p = 0; p < L16; ++p) keys[p] = (p * 7) % R16;
        for (int i = 0; i < L16 * D16; ++i) g[i] = (float)((i * 40503u) >> 4 & 0xFF) / 128.0f - 1.0f;
        if (np_ref_sparse_adagrad_16(t16, kind, s16, R16, D16, keys, g, L16, 0.01f, 1e-8f)) return 5;
        if (np_ref_sparse_adagrad(t32, s32, R16, D16, keys, g, L16, 0.01f, 1e-8f)) return 5;
        for (int r = 0; r < R16; ++r)
            if (s16[r] != s32[r]) return 5;
        const double half_spacing = kind == 1 ? ldexp(1.0, -8) : ldexp(1.0, -11);
        for (int i = 0; i < R16 * D16; ++i) {
            double a = kind == 1 ? (double)np_ref_bf16_to_f32(t16[i]) : (double)np_ref_f16_to_f32(t16[i]);
            if (fabs(a - (double)t32[i]) > fabs((double)t32[i]) * (half_spacing + 1e-6) + ldexp(1.0, -25)) return 5;
        }
    }
    return 0;
}

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
    if (check_16bit()) return 5;
    printf("oracle selftest ok\n");
    return 0;
}
