/*
 * CPU oracle for the pre-gated MoE block (arXiv 2308.12066).  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP library and to be timed as the reported CPU baseline.  It
 * shares no code with the HIP path and the product never calls it.
 *
 * The paper states the block in words, not formulas: a gate scores every expert for every
 * token with a probability, the best-scoring experts are switched on, and each of those
 * (a dense FFN) processes the tokens routed to it (Sec. II-B, MoE model architecture); the
 * pre-gate in block N produces the activation mask used by block N+1 (Sec. IV-B, Pre-gate
 * function); block 0 carries a conventional gate as well and the last block none
 * (Sec. IV-B, figure of the decoder iterations).  The numeric reading used here is the standard
 * Switch-Transformer one: softmax over x.W (+ optional bias), top-k on the logits with ties
 * to the lowest index, expert = ReLU(x.W1).W2 without biases, output = sum over the chosen
 * experts of (raw softmax probability) x (expert output), no renormalisation, no capacity
 * limit.  Everything is evaluated in fp64, straight from the definition: no blocking, no
 * fusion, no reordering.
 *
 * Weight containers: experts may be handed over as float32, as bfloat16 bit patterns or as
 * float64; element load converts to double exactly (every bf16 and f32 value is a double).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { PGO_F32 = 0, PGO_BF16 = 1, PGO_F64 = 2 };

static inline double load_elem(const void *base, size_t i, int dt) {
    if (dt == PGO_F64) return ((const double *)base)[i];
    if (dt == PGO_F32) return (double)((const float *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16; /* bf16 = top half of f32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int pgo_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Gate logits (Sec. II-B: the gate scores every expert for every token).
 * z[t,e] = sum_i x[t,i] * w[i,e] (+ bias[e]);  x [T,d], w [d,E], z [T,E], row-major. */
void pgo_gate_logits(const double *x, const double *w, const double *bias, int T, int d, int E,
                     double *z) {
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int i = 0; i < d; ++i) s += x[(size_t)t * d + i] * w[(size_t)i * E + e];
            z[(size_t)t * E + e] = s + (bias ? bias[e] : 0.0);
        }
}

/* Softmax over the experts of one token: the gate's per-expert probabilities (Sec. II-B). */
void pgo_softmax(const double *z, int T, int E, double *p) {
    for (int t = 0; t < T; ++t) {
        const double *zt = z + (size_t)t * E;
        double *pt = p + (size_t)t * E;
        double m = -INFINITY;
        for (int e = 0; e < E; ++e) if (zt[e] > m) m = zt[e];
        double s = 0.0;
        for (int e = 0; e < E; ++e) { pt[e] = exp(zt[e] - m); s += pt[e]; }
        for (int e = 0; e < E; ++e) pt[e] /= s;
    }
}

/* Top-k selection on the logits: k passes, each taking the first strict maximum among the
 * experts not taken yet, so equal logits go to the lowest index and the result is in
 * descending order.  A NaN logit ranks as -infinity and sets nan_flag[t].
 * gaps[t,j] = z_(j) - z_(j+1) for the j-th chosen value (j = 0..k-1); gaps[t,k-1] is the
 * margin between the last chosen expert and the best one left out (+inf when k == E). */
void pgo_topk(const double *z, int T, int E, int k, int32_t *idx, double *gaps, int32_t *nan_flag) {
    unsigned char *taken = (unsigned char *)malloc((size_t)E);
    double *v = (double *)malloc(sizeof(double) * (size_t)E);
    for (int t = 0; t < T; ++t) {
        int saw_nan = 0;
        for (int e = 0; e < E; ++e) {
            double a = z[(size_t)t * E + e];
            if (isnan(a)) { a = -INFINITY; saw_nan = 1; }
            v[e] = a;
            taken[e] = 0;
        }
        double prev = 0.0;
        for (int j = 0; j <= k; ++j) {           /* pass k finds the runner-up for the margin */
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!taken[e] && (best < 0 || v[e] > v[best])) best = e;
            if (j > 0) gaps[(size_t)t * k + (j - 1)] = (best >= 0) ? prev - v[best] : INFINITY;
            if (j == k || best < 0) break;
            idx[(size_t)t * k + j] = best;
            taken[best] = 1;
            prev = v[best];
        }
        if (nan_flag) nan_flag[t] = saw_nan;
    }
    free(taken);
    free(v);
}

/* Token-to-expert assignment bookkeeping (Sec. II-B: an expert processes the tokens
 * routed to it).  Entry n = t*k + j is token t's j-th choice.  counts[e] = number of entries
 * routed to e; offsets = exclusive prefix sum (offsets[E] = T*k); row_of[n] = offsets[e] +
 * (number of earlier entries n' < n with the same expert): the stable grouping by expert.
 * unique = ascending list of experts with counts > 0 (the experts that must be resident,
 * Sec. IV-C: only activated experts are migrated). */
void pgo_route(const int32_t *idx, int T, int k, int E, int32_t *counts, int32_t *offsets,
               int32_t *row_of, int32_t *unique, int32_t *n_unique) {
    *n_unique = 0;
    if (E <= 0 || T < 0 || k < 0) return;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int n = 0; n < T * k; ++n) counts[idx[n]] += 1;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t *seen = (int32_t *)calloc((size_t)E, sizeof(int32_t));
    for (int n = 0; n < T * k; ++n) {
        int e = idx[n];
        row_of[n] = offsets[e] + seen[e];
        seen[e] += 1;
    }
    free(seen);
    int u = 0;
    for (int e = 0; e < E; ++e) if (counts[e] > 0) unique[u++] = e;
    *n_unique = u;
}

/* One expert on one token: y = ReLU(x.W1).W2, W1 [d,f], W2 [f,d] row-major, no biases
 * (Sec. II-B: each expert is a dense FFN of the dense block's dimensions).  h is caller scratch of f doubles. */
static void ffn_row(const double *x, int d, int f, const void *w1, const void *w2, int dt,
                    double *h, double *y) {
    for (int j = 0; j < f; ++j) h[j] = 0.0;
    for (int i = 0; i < d; ++i) {
        const double xi = x[i];
        for (int j = 0; j < f; ++j) h[j] += xi * load_elem(w1, (size_t)i * f + j, dt);
    }
    for (int j = 0; j < f; ++j) if (!(h[j] > 0.0)) h[j] = 0.0;
    for (int c = 0; c < d; ++c) y[c] = 0.0;
    for (int j = 0; j < f; ++j) {
        const double hj = h[j];
        for (int c = 0; c < d; ++c) y[c] += hj * load_elem(w2, (size_t)j * d + c, dt);
    }
}

/* Expert outputs for n rows that all belong to one expert: y[r] = FFN(x[r]). */
void pgo_ffn_rows(const double *x, int n, int d, int f, const void *w1, const void *w2, int dt,
                  double *y, int threads) {
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
#pragma omp parallel num_threads(threads)
#endif
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)f);
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int r = 0; r < n; ++r)
            ffn_row(x + (size_t)r * d, d, f, w1, w2, dt, h, y + (size_t)r * d);
        free(h);
    }
}

/* The sparse MoE block, routed evaluation, straight from the definition:
 *   y[t] = sum_{j<k} p[t, idx[t,j]] * FFN_{idx[t,j]}(x[t]).
 * p [T,E] is the full softmax of whichever gate routes this block (the block's own gate for
 * block 0, the previous block's pre-gate otherwise) and idx [T,k] its top-k; x [T,d] is the
 * hidden state entering THIS block.  w1[e] / w2[e] may be NULL for experts no token chose.
 * Returns 0, or -1 if a chosen expert has no weights. */
int pgo_block(const double *x, const double *p, const int32_t *idx, int T, int d, int f, int E,
              int k, const void *const *w1, const void *const *w2, int dt, double *y, int threads) {
    for (int n = 0; n < T * k; ++n) {
        int e = idx[n];
        if (e < 0 || e >= E || !w1[e] || !w2[e]) return -1;
    }
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
#pragma omp parallel num_threads(threads)
#endif
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)f);
        double *ye = (double *)malloc(sizeof(double) * (size_t)d);
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int t = 0; t < T; ++t) {
            double *yt = y + (size_t)t * d;
            for (int c = 0; c < d; ++c) yt[c] = 0.0;
            for (int j = 0; j < k; ++j) {
                int e = idx[(size_t)t * k + j];
                ffn_row(x + (size_t)t * d, d, f, w1[e], w2[e], dt, h, ye);
                const double pe = p[(size_t)t * E + e];
                for (int c = 0; c < d; ++c) yt[c] += pe * ye[c];
            }
        }
        free(h);
        free(ye);
    }
    return 0;
}
