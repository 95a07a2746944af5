/* Runs the C oracle's functions on small seeded inputs, edge cases included, under AddressSanitizer
 * and UndefinedBehaviorSanitizer (built by tests/test_sanitize.py from oracle/emoe_oracle.c with gcc).
 * The values are pinned elsewhere (tests/test_oracle_pins.py); here only invariants that need no
 * second implementation are checked, the point being that every loop runs with the sanitizers on. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_gate_logits(int T, int d, int E, int dtype, const void *x, const void *w_gate, const float *gate_bias,
                       double *logits);
int oracle_route_mask_then_topk(int T, int E, int k, const double *logits, const int32_t *slot_of_expert, int32_t *idx,
                                double *w);
int oracle_route_rank_then_skip(int T, int E, int k, const double *logits, const int32_t *slot_of_expert, int32_t *idx,
                                double *w);
int oracle_route_unrestricted(int T, int E, int k, const double *logits, int32_t *idx);
int oracle_permute(int T, int k, int E, int S, const int32_t *idx, const int32_t *slot_of_expert, int32_t *counts,
                   int32_t *offsets, int32_t *perm, int32_t *inv_perm);
int oracle_gather_rows(int A, int k, int d, int dtype, const void *x, const int32_t *perm, void *out);
int oracle_expert_ffn_rows(int n, const int32_t *row_token, const int32_t *row_slot, int d, int f, int act, int dtype,
                           const void *x, const void *w1, const void *w3, const void *w2, double *y, double *h);
int oracle_combine_tokens(int n, const int32_t *tokens, int k, int d, const double *w, const int32_t *row_index,
                          const double *y_rows, double *out);

static uint64_t state = 2503068230ull;
static uint32_t rnd(void) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}
static float rfloat(void) { return (float)((int)(rnd() % 2001) - 1000) / 500.0f; }
static uint16_t bf16_of(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)(u >> 16); } /* truncation: any bf16 will do */

#define REQUIRE(c) do { if (!(c)) { fprintf(stderr, "%s:%d: %s failed\n", __FILE__, __LINE__, #c); exit(1); } } while (0)

static void *fill(size_t n, int dtype) {
    void *p = malloc(n * (dtype ? 2 : 4) + 1);
    for (size_t i = 0; i < n; ++i) {
        if (dtype) ((uint16_t *)p)[i] = bf16_of(rfloat());
        else ((float *)p)[i] = rfloat();
    }
    return p;
}

static void one_layer(int T, int d, int f, int E, int k, int R, int S, int dtype, int act, int with_bias) {
    const int A = T * k;
    void *x = fill((size_t)T * d, dtype), *wg = fill((size_t)E * d, dtype);
    void *w1 = fill((size_t)S * f * d, dtype), *w3 = act == 0 ? fill((size_t)S * f * d, dtype) : NULL;
    void *w2 = fill((size_t)S * d * f, dtype);
    float *bias = NULL;
    if (with_bias) { bias = malloc(sizeof(float) * E); for (int e = 0; e < E; ++e) bias[e] = rfloat(); }
    int32_t *soe = malloc(sizeof(int32_t) * E);
    for (int e = 0; e < E; ++e) soe[e] = -1;
    for (int r = 0; r < R;) { int e = rnd() % E; if (soe[e] < 0) { soe[e] = 0; ++r; } }
    { /* distinct slots: the residents take consecutive slots from a random start, wrapping around */
        int s = rnd() % S, n = 0;
        for (int e = 0; e < E; ++e) if (soe[e] >= 0) { soe[e] = (s + n) % S; ++n; }
    }
    double *lg = malloc(sizeof(double) * (T * E + 1));
    REQUIRE(oracle_gate_logits(T, d, E, dtype, x, wg, bias, lg) == 0);
    int32_t *idx = malloc(sizeof(int32_t) * (A + 1)), *idx2 = malloc(sizeof(int32_t) * (A + 1));
    double *w = malloc(sizeof(double) * (A + 1)), *wb = malloc(sizeof(double) * (A + 1));
    REQUIRE(oracle_route_mask_then_topk(T, E, k, lg, soe, idx, w) == 0);
    REQUIRE(oracle_route_rank_then_skip(T, E, k, lg, soe, idx2, wb) == 0);
    REQUIRE(memcmp(idx, idx2, sizeof(int32_t) * A) == 0);
    for (int t = 0; t < T; ++t) {
        double sum = 0;
        for (int j = 0; j < k; ++j) { REQUIRE(soe[idx[t * k + j]] >= 0); sum += w[t * k + j]; }
        REQUIRE(fabs(sum - 1.0) < 1e-12);
    }
    REQUIRE(oracle_route_unrestricted(T, E, k, lg, idx2) == 0);
    int32_t *counts = malloc(sizeof(int32_t) * S), *offsets = malloc(sizeof(int32_t) * (S + 1));
    int32_t *perm = malloc(sizeof(int32_t) * (A + 1)), *inv = malloc(sizeof(int32_t) * (A + 1));
    REQUIRE(oracle_permute(T, k, E, S, idx, soe, counts, offsets, perm, inv) == 0);
    REQUIRE(offsets[S] == A);
    for (int r = 0; r < A; ++r) REQUIRE(inv[perm[r]] == r);
    void *xp = malloc((size_t)A * d * (dtype ? 2 : 4) + 1);
    REQUIRE(oracle_gather_rows(A, k, d, dtype, x, perm, xp) == 0);
    int32_t *row_token = malloc(sizeof(int32_t) * (A + 1)), *row_slot = malloc(sizeof(int32_t) * (A + 1));
    for (int r = 0; r < A; ++r) { row_token[r] = perm[r] / k; row_slot[r] = soe[idx[perm[r]]]; }
    double *y = malloc(sizeof(double) * ((size_t)A * d + 1)), *h = malloc(sizeof(double) * ((size_t)A * f + 1));
    REQUIRE(oracle_expert_ffn_rows(A, row_token, row_slot, d, f, act, dtype, x, w1, w3, w2, y, h) == 0);
    REQUIRE(oracle_expert_ffn_rows(A, row_token, row_slot, d, f, act, dtype, x, w1, w3, w2, y, NULL) == 0);
    for (size_t i = 0; i < (size_t)A * d; ++i) REQUIRE(isfinite(y[i]));
    int32_t *tokens = malloc(sizeof(int32_t) * (T + 1)), *row_index = malloc(sizeof(int32_t) * (A + 1));
    for (int t = 0; t < T; ++t) { tokens[t] = t; for (int j = 0; j < k; ++j) row_index[t * k + j] = inv[t * k + j]; }
    double *out = malloc(sizeof(double) * ((size_t)T * d + 1));
    REQUIRE(oracle_combine_tokens(T, tokens, k, d, w, row_index, y, out) == 0);
    /* fewer than k resident experts is an error, not an out-of-bounds walk */
    if (R < E && T > 0) {
        int32_t *none = malloc(sizeof(int32_t) * E);
        for (int e = 0; e < E; ++e) none[e] = -1;
        if (k > 1) none[0] = 0;
        REQUIRE(oracle_route_mask_then_topk(T, E, k, lg, none, idx, w) != 0);
        REQUIRE(oracle_route_rank_then_skip(T, E, k, lg, none, idx, w) != 0);
        free(none);
    }
    free(x); free(wg); free(w1); free(w3); free(w2); free(bias); free(soe); free(lg); free(idx); free(idx2); free(w);
    free(wb); free(counts); free(offsets); free(perm); free(inv); free(xp); free(row_token); free(row_slot); free(y);
    free(h); free(tokens); free(row_index); free(out);
}

int main(void) {
    one_layer(64, 128, 256, 8, 2, 4, 4, 0, 0, 0);      /* the tiny fp32 workload's shape */
    one_layer(0, 16, 24, 4, 1, 2, 3, 1, 1, 1);         /* no tokens */
    one_layer(1, 8, 8, 1, 1, 1, 1, 1, 0, 0);           /* one token, one expert */
    one_layer(37, 24, 40, 64, 6, 24, 30, 1, 0, 1);     /* top-6 of 24 resident among 64, more slots than residents */
    one_layer(50, 16, 8, 6, 3, 3, 6, 0, 1, 0);         /* k = R */
    for (int i = 0; i < 40; ++i) {
        const int E = 1 + rnd() % 32, R = 1 + rnd() % E, k = 1 + rnd() % (R < 6 ? R : 6), S = R + rnd() % (E - R + 1);
        one_layer(rnd() % 70, 8 * (1 + rnd() % 6), 8 * (1 + rnd() % 9), E, k, R, S, rnd() % 2, rnd() % 2, rnd() % 2);
    }
    printf("oracle driver: ok\n");
    return 0;
}
