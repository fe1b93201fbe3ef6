/*
 * CPU oracle for the sparse MoE layer (TEST INFRASTRUCTURE, not product code).
 *
 * This file is the plain definition of what the GPU library computes, written
 * token by token in fp64.  It shares nothing with the HIP path: no headers, no
 * helpers, no tables.  Only tests, the smoke check and the benchmark's CPU
 * baseline leg may build or call it.
 *
 * What it follows (DAOP paper, arXiv 2501.10375):
 *   - Sec. II-A "MoE Structure": a gating function scores every expert for a
 *     token's hidden state; the top-k experts are selected and transform the
 *     token.  The paper builds on Mixtral 8x7B (Sec. I, Table III), whose
 *     public definition fixes the details the paper does not spell out: the
 *     gate is one linear map H->E followed by a softmax over all E experts,
 *     the k largest probabilities are renormalised to sum to one, and an
 *     expert is the SwiGLU network  W2 ( silu(W1 x) * (W3 x) ).
 *   - Sec. IV-B and Algorithm 1 (the two "active experts" steps): the activity
 *     level of an expert is the number of the sequence's tokens routed to it.
 *   - Sec. III observation 3 / Sec. IV-C "Accuracy Stabilization": next-layer
 *     experts are predicted by applying the next layer's gate to the very same
 *     hidden state the current layer's gate sees.
 *
 * Precision: inputs are taken in their storage type (fp32, bf16 bit patterns,
 * or fp64) and widened exactly to double; every sum is a double running sum in
 * index order; nothing is rounded on the way except where fp32 semantics are
 * part of the definition of the routing decision (see oracle_route).
 *
 * Pins (tests/test_oracle_*.py): brute force on dyadic tiny inputs, the
 * softmax-over-selected closed form, zero-input and single-expert special
 * cases, E=1 dense SwiGLU and k=E soft mixture against a library matmul,
 * homogeneity, token independence, expert-permutation equivariance, and the
 * count invariants; the pre-calculation variant against the pinned expert
 * function (identical inputs, all-fresh, all-stale, and its linearity in the
 * combine weights).  No function here is "parity unpinned".
 * tests/test_oracle_mutants.py plants mistakes in a copy of this file, one
 * expression at a time, and requires each to fail a pin; it finds the
 * expressions by their text, so it says so when an edit here moves them.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

/* Exact widening of one stored element to double. */
static double load_elem(const void *base, int dtype, size_t i) {
    if (dtype == ORACLE_F32) return (double)((const float *)base)[i];
    if (dtype == ORACLE_F64) return ((const double *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16; /* bf16 = top half of fp32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* sum_i row[i] * v[i], running double sum in index order. */
static double dot_row(const void *mat, int dtype, size_t row_offset, const double *v, int n) {
    double s = 0.0;
    if (dtype == ORACLE_F32) {
        const float *r = (const float *)mat + row_offset;
        for (int i = 0; i < n; ++i) s += (double)r[i] * v[i];
    } else if (dtype == ORACLE_F64) {
        const double *r = (const double *)mat + row_offset;
        for (int i = 0; i < n; ++i) s += r[i] * v[i];
    } else {
        const uint16_t *r = (const uint16_t *)mat + row_offset;
        for (int i = 0; i < n; ++i) {
            uint32_t bits = (uint32_t)r[i] << 16;
            float f;
            memcpy(&f, &bits, sizeof f);
            s += (double)f * v[i];
        }
    }
    return s;
}

/*
 * Gate + softmax + top-k + renormalise + activation counts for T tokens.
 *
 *   z[e]  = sum_h x[t,h] * wg[e,h] + bias[e]         (double), then z32 = (float) z
 *   p[e]  = exp(z32[e] - max z32) / sum_e' exp(z32[e'] - max z32)   evaluated in
 *           double on the fp32 logits, then rounded once to fp32
 *   idx   = experts ordered by p descending, equal p -> lower expert index
 *           first; the first k are selected
 *   w[j]  = p[idx_j] / sum_j' p[idx_j']
 *   counts[idx_j] += 1
 *
 * The routing decision is taken on fp32 probabilities because that is the
 * precision the GPU decides in; everything before the cast is fp64.
 *
 * margin[t] = min over r = 1..k of (p_(r) - p_(r+1)) on the sorted fp32
 * probabilities (for k == E the last term does not exist and is dropped): the
 * smallest gap whose sign decides either the selected set or its order.
 *
 * x [T,H], wg [E,H] in `dtype`; bias [E] double or NULL.
 * idx [T,k] int32, w [T,k] double, probs [T,E] float or NULL,
 * margin [T] float or NULL, counts [E] int32 (zeroed first unless accumulate).
 * Returns 0, or -1 on a bad argument.
 */
int oracle_route(int T, int H, int E, int k, int dtype, const void *x, const void *wg,
                 const double *bias, int32_t *idx, double *w, float *probs, float *margin,
                 int32_t *counts, int accumulate) {
    if (T < 0 || H <= 0 || E <= 0 || k <= 0 || k > E) return -1;
    if (counts && !accumulate)
        for (int e = 0; e < E; ++e) counts[e] = 0;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double *xt = (double *)malloc(sizeof(double) * (size_t)H);
        float *p32 = (float *)malloc(sizeof(float) * (size_t)E);
        float *z32 = (float *)malloc(sizeof(float) * (size_t)E);
        int *order = (int *)malloc(sizeof(int) * (size_t)E);
        if (!xt || !p32 || !z32 || !order) {
            bad = 1;
        } else {
            for (int h = 0; h < H; ++h) xt[h] = load_elem(x, dtype, (size_t)t * H + h);
            for (int e = 0; e < E; ++e) {
                double z = dot_row(wg, dtype, (size_t)e * H, xt, H);
                if (bias) z += bias[e];
                z32[e] = (float)z;
            }
            float zmax = z32[0];
            for (int e = 1; e < E; ++e)
                if (z32[e] > zmax) zmax = z32[e];
            double denom = 0.0;
            for (int e = 0; e < E; ++e) denom += exp((double)z32[e] - (double)zmax);
            for (int e = 0; e < E; ++e)
                p32[e] = (float)(exp((double)z32[e] - (double)zmax) / denom);
            /* Full ordering by insertion: descending p, ties keep the lower index first. */
            for (int e = 0; e < E; ++e) {
                int pos = e;
                while (pos > 0 && p32[order[pos - 1]] < p32[e]) {
                    order[pos] = order[pos - 1];
                    --pos;
                }
                order[pos] = e;
            }
            double wsum = 0.0;
            for (int j = 0; j < k; ++j) wsum += (double)p32[order[j]];
            for (int j = 0; j < k; ++j) {
                idx[(size_t)t * k + j] = order[j];
                w[(size_t)t * k + j] = (double)p32[order[j]] / wsum;
            }
            if (probs)
                for (int e = 0; e < E; ++e) probs[(size_t)t * E + e] = p32[e];
            if (margin) {
                int last = (k < E) ? k : E - 1; /* gaps r = 1..last */
                float m = INFINITY;
                for (int r = 0; r < last; ++r) {
                    float gap = p32[order[r]] - p32[order[r + 1]];
                    if (gap < m) m = gap;
                }
                margin[t] = m;
            }
        }
        free(xt);
        free(p32);
        free(z32);
        free(order);
    }
    if (bad) return -1;
    /* Integer histogram of the selections, in token order. */
    if (counts)
        for (int t = 0; t < T; ++t)
            for (int j = 0; j < k; ++j) counts[idx[(size_t)t * k + j]] += 1;
    return 0;
}

/*
 * Expert execution and weighted combine for a list of tokens.
 *
 * For token t with selections (e_j, w_j), j = 0..k-1:
 *   g[f] = sum_h w1[e_j,f,h] x[t,h]      u[f] = sum_h w3[e_j,f,h] x[t,h]
 *   a[f] = silu(g[f]) * u[f],            silu(z) = z / (1 + exp(-z))
 *   o[h] = sum_f w2[e_j,h,f] a[f]
 *   y[t,h] = sum_j w_j o_j[h]            (j ascending)
 * All in double, nothing rounded.
 *
 * x [T,H]; idx [T,k]; w [T,k] double; w1,w3 [E,F,H]; w2 [E,H,F] in `dtype`.
 * tokens: ns token indices (or NULL meaning 0..ns-1); y [ns,H] double, row i
 * holding the output for tokens[i].  Returns 0, or -1 on a bad argument.
 */
int oracle_expert_ffn(int T, int H, int F, int E, int k, int dtype, const void *x,
                      const int32_t *idx, const double *w, const void *w1, const void *w3,
                      const void *w2, const int32_t *tokens, int ns, double *y) {
    if (T < 0 || H <= 0 || F <= 0 || E <= 0 || k <= 0 || k > E || ns < 0) return -1;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < ns; ++i) {
        int t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) {
            bad = 1;
            continue;
        }
        double *xt = (double *)malloc(sizeof(double) * (size_t)H);
        double *a = (double *)malloc(sizeof(double) * (size_t)F);
        if (!xt || !a) {
            bad = 1;
            free(xt);
            free(a);
            continue;
        }
        for (int h = 0; h < H; ++h) xt[h] = load_elem(x, dtype, (size_t)t * H + h);
        for (int h = 0; h < H; ++h) y[(size_t)i * H + h] = 0.0;
        for (int j = 0; j < k; ++j) {
            int e = idx[(size_t)t * k + j];
            if (e < 0 || e >= E) {
                bad = 1;
                break;
            }
            for (int f = 0; f < F; ++f) {
                size_t row = ((size_t)e * F + f) * (size_t)H;
                double g = dot_row(w1, dtype, row, xt, H);
                double u = dot_row(w3, dtype, row, xt, H);
                a[f] = g / (1.0 + exp(-g)) * u;
            }
            double wj = w[(size_t)t * k + j];
            for (int h = 0; h < H; ++h) {
                size_t row = ((size_t)e * H + h) * (size_t)F;
                y[(size_t)i * H + h] += wj * dot_row(w2, dtype, row, a, F);
            }
        }
        free(xt);
        free(a);
    }
    return bad ? -1 : 0;
}

/*
 * Expert execution with pre-calculated experts (Sec. IV-C "Prediction-based
 * Expert Pre-Calculation"): an expert of block i+1 that was predicted one block
 * ahead and does not sit on the GPU has already been started on the hidden
 * state block i worked on, so its input is that earlier ("stale") state; every
 * other selected expert sees the block's true input.  Per selection (t, j):
 *
 *   in(t, j) = stale[t,j] ? x_stale[t] : x[t]
 *   y[t]     = sum_j w[t,j] * W2_e ( silu(W1_e in(t,j)) * (W3_e in(t,j)) ),  e = idx[t,j]
 *
 * stale: uint8 [T,k], non-zero = the selection was evaluated on x_stale.  The
 * paper gives no formula; this is its description written out, with the combine
 * weights supplied by the caller (it does not say whether the predicted or the
 * actual gate's weights apply).  Other arguments as in oracle_expert_ffn.
 */
int oracle_expert_ffn_precalc(int T, int H, int F, int E, int k, int dtype, const void *x,
                              const void *x_stale, const uint8_t *stale, const int32_t *idx,
                              const double *w, const void *w1, const void *w3, const void *w2,
                              const int32_t *tokens, int ns, double *y) {
    if (T < 0 || H <= 0 || F <= 0 || E <= 0 || k <= 0 || k > E || ns < 0) return -1;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < ns; ++i) {
        int t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) {
            bad = 1;
            continue;
        }
        double *in = (double *)malloc(sizeof(double) * (size_t)H);
        double *hid = (double *)malloc(sizeof(double) * (size_t)F);
        if (!in || !hid) {
            bad = 1;
            free(in);
            free(hid);
            continue;
        }
        double *yt = y + (size_t)i * H;
        for (int h = 0; h < H; ++h) yt[h] = 0.0;
        for (int j = 0; j < k; ++j) {
            size_t sel = (size_t)t * k + j;
            int e = idx[sel];
            if (e < 0 || e >= E) {
                bad = 1;
                break;
            }
            const void *source = stale[sel] ? x_stale : x;
            for (int h = 0; h < H; ++h) in[h] = load_elem(source, dtype, (size_t)t * H + h);
            for (int f = 0; f < F; ++f) {
                size_t wrow = ((size_t)e * F + f) * (size_t)H;
                double gate = dot_row(w1, dtype, wrow, in, H);
                double up = dot_row(w3, dtype, wrow, in, H);
                hid[f] = gate / (1.0 + exp(-gate)) * up;
            }
            for (int h = 0; h < H; ++h)
                yt[h] += w[sel] * dot_row(w2, dtype, ((size_t)e * H + h) * (size_t)F, hid, F);
        }
        free(in);
        free(hid);
    }
    return bad ? -1 : 0;
}

/* Number of worker threads the parallel loops above will use. */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) {
    if (n > 0) omp_set_num_threads(n);
}
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
