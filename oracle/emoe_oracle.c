/*
 * TEST INFRASTRUCTURE -- not part of the product.
 *
 * Plain fp64 CPU oracle for one MoE layer forward restricted to the experts
 * resident on the GPU (eMoE, arxiv 2503.06823).  Slow and literal on purpose:
 * no blocking, no fusion, no reordering beyond the definitions below.  It
 * shares no code with the HIP library and is called only from tests, the smoke
 * check and the benchmark's cpu_baseline leg.
 *
 * What the paper fixes (Section 3.2.2, last paragraph): when the expert chosen
 * for a token is not resident, the token goes to its next-best expert that is.
 * The layer itself is the usual gate-plus-experts block (Section 1) of the
 * models the paper serves (Section 2.1).  Readings taken where the paper is
 * silent:
 *   - every token always gets exactly k resident experts (absent ones are
 *     replaced, not dropped); fewer than k resident experts is an error;
 *   - the k experts are listed by descending logit, ties to the lower index;
 *   - gate weights are the softmax over the k selected logits (sum to 1);
 *   - rows are grouped by slot id, inside a slot by ascending assignment
 *     index a = t*k + j (stable);
 *   - SwiGLU: h = silu(W1 x) * (W3 x), y = W2 h;  ReLU: h = max(W1 x, 0),
 *     y = W2 h;  no biases in the experts.
 *
 * Inputs arrive in their storage type (fp32, or bf16 as uint16 bit patterns)
 * and are widened exactly to double; nothing is rounded on the way.
 *
 * Pins (tests/test_oracle_pins.py): weights sum to one and decrease; resident
 * only; all-resident == textbook softmax->top-k->renormalise; E=1 == dense
 * FFN by numpy matmul; k=R == dense mixture; both routing formulations agree;
 * permutation == brute-force lists; token-permutation equivariance;
 * slot-relabel invariance; scalar closed form 6/(1+e^-1); homogeneity in W2;
 * miss accounting.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_SWIGLU = 0, ORACLE_RELU = 1 };
enum { ORACLE_OK = 0, ORACLE_ERR_ARG = -1, ORACLE_ERR_RESIDENT = -4 };

/* exact widening of element i of a storage array */
static double widen(const void *base, size_t i, int dtype) {
    if (dtype == ORACLE_F32) return (double)((const float *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* O1: l[t,e] = sum_i x[t,i] * Wg[e,i] + b[e], for all E experts. */
int oracle_gate_logits(int T, int d, int E, int dtype, const void *x, const void *w_gate,
                       const float *gate_bias, double *logits) {
    if (T < 0 || d <= 0 || E <= 0) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int i = 0; i < d; ++i)
                acc += widen(x, (size_t)t * d + i, dtype) * widen(w_gate, (size_t)e * d + i, dtype);
            if (gate_bias) acc += (double)gate_bias[e];
            logits[(size_t)t * E + e] = acc;
        }
    }
    return ORACLE_OK;
}

/* O3: softmax over the k selected logits, shifted by the largest. */
static void selected_softmax(const double *l, const int32_t *idx, int k, double *w) {
    double m = l[idx[0]];
    double sum = 0.0;
    for (int j = 0; j < k; ++j) {
        w[j] = exp(l[idx[j]] - m);
        sum += w[j];
    }
    for (int j = 0; j < k; ++j) w[j] /= sum;
}

static int count_resident(int E, const int32_t *slot_of_expert) {
    int n = 0;
    for (int e = 0; e < E; ++e) n += slot_of_expert[e] >= 0;
    return n;
}

/* O2, formulation A: absent experts are masked out, then the k best of what
 * is left are taken one by one (largest logit, lower index on ties). */
int oracle_route_mask_then_topk(int T, int E, int k, const double *logits, const int32_t *slot_of_expert,
                                int32_t *idx, double *w) {
    if (T < 0 || E <= 0 || k <= 0) return ORACLE_ERR_ARG;
    if (count_resident(E, slot_of_expert) < k) return ORACLE_ERR_RESIDENT;
    char *taken = (char *)malloc((size_t)E);
    if (!taken) return ORACLE_ERR_ARG;
    for (int t = 0; t < T; ++t) {
        const double *l = logits + (size_t)t * E;
        for (int e = 0; e < E; ++e) taken[e] = slot_of_expert[e] < 0; /* masked == never eligible */
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e; /* strict > keeps the lower index on ties */
            }
            taken[best] = 1;
            idx[(size_t)t * k + j] = best;
        }
        selected_softmax(l, idx + (size_t)t * k, k, w + (size_t)t * k);
    }
    free(taken);
    return ORACLE_OK;
}

/* O2, formulation B (the paper's wording): rank ALL experts as the unrestricted
 * gate would, walk the ranking downwards and skip experts that are not resident. */
int oracle_route_rank_then_skip(int T, int E, int k, const double *logits, const int32_t *slot_of_expert,
                                int32_t *idx, double *w) {
    if (T < 0 || E <= 0 || k <= 0) return ORACLE_ERR_ARG;
    if (count_resident(E, slot_of_expert) < k) return ORACLE_ERR_RESIDENT;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    if (!order) return ORACLE_ERR_ARG;
    for (int t = 0; t < T; ++t) {
        const double *l = logits + (size_t)t * E;
        /* insertion sort by (logit descending, index ascending) */
        for (int e = 0; e < E; ++e) {
            int p = e;
            while (p > 0 && l[order[p - 1]] < l[e]) {
                order[p] = order[p - 1];
                --p;
            }
            order[p] = e;
        }
        int j = 0;
        for (int r = 0; r < E && j < k; ++r)
            if (slot_of_expert[order[r]] >= 0) idx[(size_t)t * k + j++] = order[r];
        selected_softmax(l, idx + (size_t)t * k, k, w + (size_t)t * k);
    }
    free(order);
    return ORACLE_OK;
}

/* Unrestricted top-k of the ordinary gate (used for miss accounting only). */
int oracle_route_unrestricted(int T, int E, int k, const double *logits, int32_t *idx) {
    if (T < 0 || E <= 0 || k <= 0 || k > E) return ORACLE_ERR_ARG;
    int32_t *all = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    double *w = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * k);
    if (!all || !w) { free(all); free(w); return ORACLE_ERR_ARG; }
    for (int e = 0; e < E; ++e) all[e] = e; /* every expert "resident" */
    int rc = oracle_route_mask_then_topk(T, E, k, logits, all, idx, w);
    free(all);
    free(w);
    return rc;
}

/* O4: stable grouping of the A = T*k assignments by slot id.
 * perm[r] = assignment placed in row r; inv_perm[a] = row of assignment a;
 * counts[s] rows in slot s; offsets = exclusive scan of counts (length S+1). */
int oracle_permute(int T, int k, int E, int S, const int32_t *idx, const int32_t *slot_of_expert,
                   int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm) {
    if (T < 0 || k <= 0 || E <= 0 || S <= 0) return ORACLE_ERR_ARG;
    const int A = T * k;
    int r = 0;
    for (int s = 0; s < S; ++s) {
        offsets[s] = r;
        counts[s] = 0;
        for (int a = 0; a < A; ++a) {
            int e = idx[a];
            if (e < 0 || e >= E) return ORACLE_ERR_ARG;
            int key = slot_of_expert[e];
            if (key < 0 || key >= S) return ORACLE_ERR_RESIDENT;
            if (key == s) {
                perm[r] = a;
                inv_perm[a] = r;
                ++r;
                ++counts[s];
            }
        }
    }
    offsets[S] = r;
    return r == A ? ORACLE_OK : ORACLE_ERR_ARG;
}

/* x_perm[r,:] = x[perm[r] / k, :] -- a copy in storage type. */
int oracle_gather_rows(int A, int k, int d, int dtype, const void *x, const int32_t *perm, void *x_perm) {
    size_t row_bytes = (size_t)d * (dtype == ORACLE_F32 ? 4 : 2);
    for (int r = 0; r < A; ++r)
        memcpy((char *)x_perm + (size_t)r * row_bytes, (const char *)x + (size_t)(perm[r] / k) * row_bytes,
               row_bytes);
    return ORACLE_OK;
}

/* O5 for a list of rows: row n uses token row_token[n] and the weights in slot row_slot[n].
 * y is [n_rows, d] double; h_out (optional) is [n_rows, f] double. */
int oracle_expert_ffn_rows(int n_rows, const int32_t *row_token, const int32_t *row_slot, int d, int f,
                           int act, int dtype, const void *x, const void *w1_slots, const void *w3_slots,
                           const void *w2_slots, double *y, double *h_out) {
    if (n_rows < 0 || d <= 0 || f <= 0) return ORACLE_ERR_ARG;
    if (act == ORACLE_SWIGLU && !w3_slots) return ORACLE_ERR_ARG;
    double *h = (double *)malloc(sizeof(double) * (size_t)f);
    if (!h) return ORACLE_ERR_ARG;
    for (int n = 0; n < n_rows; ++n) {
        const size_t xo = (size_t)row_token[n] * d;
        const size_t w13 = (size_t)row_slot[n] * f * d; /* start of this slot's [f,d] matrix */
        const size_t w2o = (size_t)row_slot[n] * d * f; /* start of this slot's [d,f] matrix */
#pragma omp parallel for schedule(static)
        for (int i = 0; i < f; ++i) {
            double g = 0.0;
            for (int c = 0; c < d; ++c) g += widen(w1_slots, w13 + (size_t)i * d + c, dtype) * widen(x, xo + c, dtype);
            if (act == ORACLE_SWIGLU) {
                double u = 0.0;
                for (int c = 0; c < d; ++c)
                    u += widen(w3_slots, w13 + (size_t)i * d + c, dtype) * widen(x, xo + c, dtype);
                h[i] = (g / (1.0 + exp(-g))) * u;
            } else {
                h[i] = g > 0.0 ? g : 0.0;
            }
        }
        if (h_out) memcpy(h_out + (size_t)n * f, h, sizeof(double) * (size_t)f);
#pragma omp parallel for schedule(static)
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int i = 0; i < f; ++i) acc += widen(w2_slots, w2o + (size_t)j * f + i, dtype) * h[i];
            y[(size_t)n * d + j] = acc;
        }
    }
    free(h);
    return ORACLE_OK;
}

/* O6 for a list of tokens: out[n,:] = sum_j w[t,j] * y_rows[row_index[n*k+j], :], j ascending.
 * row_index maps (token n of the list, j) to a row of the y array passed in. */
int oracle_combine_tokens(int n_tokens, const int32_t *tokens, int k, int d, const double *w,
                          const int32_t *row_index, const double *y_rows, double *out) {
    for (int n = 0; n < n_tokens; ++n) {
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j)
                acc += w[(size_t)tokens[n] * k + j] * y_rows[(size_t)row_index[(size_t)n * k + j] * d + c];
            out[(size_t)n * d + c] = acc;
        }
    }
    return ORACLE_OK;
}

/* Number of threads for the loops over independent rows (timing of the oracle as a baseline only:
 * the results do not depend on it). */
int oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
    return ORACLE_OK;
}

int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
