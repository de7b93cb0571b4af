/*
 * CPU oracle for the dynamically gated Mixture-of-Experts layer forward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition the GPU
 * library is checked against.  It shares no code, header, table or helper with
 * the HIP path, and nothing on the product path may call it.
 *
 * What is defined here (paper: "Towards MoE Deployment: Mitigating
 * Inefficiencies in Mixture-of-Expert (MoE) Inference"):
 *   - the gate is a linear layer over the token vector (Sec. 2.4, "Expert
 *     Parallelism": the gating function is a lightweight linear layer);
 *   - every token goes to its top-k experts, k = 1 or 2 in the paper (Sec. 2.3);
 *   - dynamic gating (Sec. 5.1, "Case for Dynamic Gating"): sort the expert
 *     assignments, count the occurrences of each expert, reorder the inputs by
 *     the sort index, split them by the counts; no token is dropped and no
 *     placeholder row exists; after the experts, rows go back to their original
 *     order by indexing;
 *   - static gating (Sec. 3.2 and Sec. 5.1): every expert has a fixed number of
 *     rows; a token takes the first empty row of its expert, is dropped when
 *     none is left, and unused rows stay zero.
 *
 * Arithmetic: inputs are fp32 values (dt = 0) or bf16 bit patterns (dt = 1,
 * widened exactly); every sum is accumulated in fp64 (dot products in a few partial sums, see dot_ff); nothing is
 * rounded between the steps except the gate logits, which are rounded once to
 * fp32 because the top-k decision is specified on fp32 logits (both sides take
 * the integer decision in the same precision).
 *
 * Conventions the paper leaves open (listed with their reasons in the design
 * notes of this repository): softmax over the expert logits; selection on the
 * logits; ties go to the lowest expert index; slot 0 is the largest logit;
 * renorm = 1 normalises the k selected probabilities to sum to 1; rows inside
 * an expert's batch are in ascending token order; FFN = W2 * relu(W1 x + b1) + b2
 * with W1 [E,F,D], W2 [E,D,F] row-major.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline double ld(const void *p, size_t i, int dt)
{
    if (dt == 0)
        return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* sum_i a[i] * b[i] in fp64.  Every term is an exact fp64 product of two fp32 / bf16 values; the simd
 * clause lets the compiler keep several partial sums, so the ADDITION order is not the index order (a
 * comment-only correction: the arithmetic is unchanged; in fp64 the order moves a sum of 2048..8192 such
 * terms by about 1e-16 relative, far below the fp32 rounding of the logits and every tolerance). */
static double dot_ff(const float *a, const float *b, int n)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int i = 0; i < n; ++i)
        acc += (double)a[i] * (double)b[i];
    return acc;
}

static double dot_df(const double *a, const float *b, int n)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int i = 0; i < n; ++i)
        acc += a[i] * (double)b[i];
    return acc;
}

static inline float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static double dot_fb(const float *a, const uint16_t *b, int n)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int i = 0; i < n; ++i)
        acc += (double)a[i] * (double)bf16_to_f32(b[i]);
    return acc;
}

static double dot_bb(const uint16_t *a, const uint16_t *b, int n)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int i = 0; i < n; ++i)
        acc += (double)bf16_to_f32(a[i]) * (double)bf16_to_f32(b[i]);
    return acc;
}

static double dot_db(const double *a, const uint16_t *b, int n)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int i = 0; i < n; ++i)
        acc += a[i] * (double)bf16_to_f32(b[i]);
    return acc;
}

/* Gate (Sec. 2.4): logits[t,e] = sum_d x[t,d] * wg[e,d] + bias[e], fp64 sum, one
 * rounding to fp32.  x [T,D], wg [E,D] in storage type dt; bias fp32 or NULL. */
void moe_oracle_gate_logits(const void *x, const void *wg, const float *bias,
                            int T, int D, int E, int dt, float *logits)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double acc = dt == 0 ? dot_ff((const float *)x + (size_t)t * D, (const float *)wg + (size_t)e * D, D)
                                 : dot_bb((const uint16_t *)x + (size_t)t * D, (const uint16_t *)wg + (size_t)e * D, D);
            if (bias)
                acc += (double)bias[e];
            logits[(size_t)t * E + e] = (float)acc;
        }
    }
}

/* Top-k gating (Sec. 2.3).  For every token pick the k experts with the largest
 * fp32 logit, slot 0 the largest; equal logits go to the lower expert index.
 * Gate weights from the softmax of the logits, in fp64:
 *   renorm = 1: w[t,j] = exp(l_j - m) / sum over the k selected of exp(l - m)
 *   renorm = 0: w[t,j] = exp(l_j - m) / sum over all E experts of exp(l - m)
 * with m the largest logit of the token. */
void moe_oracle_topk(const float *logits, int T, int E, int k, int renorm,
                     int32_t *idx, double *w)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *l = logits + (size_t)t * E;
        int32_t *sel = idx + (size_t)t * k;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                int taken = 0;
                for (int q = 0; q < j; ++q)
                    if (sel[q] == e)
                        taken = 1;
                if (taken)
                    continue;
                if (best < 0 || l[e] > l[best])
                    best = e;
            }
            sel[j] = best;
        }
        double m = (double)l[sel[0]];
        double denom = 0.0;
        if (renorm) {
            for (int j = 0; j < k; ++j)
                denom += exp((double)l[sel[j]] - m);
        } else {
            for (int e = 0; e < E; ++e)
                denom += exp((double)l[e] - m);
        }
        for (int j = 0; j < k; ++j)
            w[(size_t)t * k + j] = exp((double)l[sel[j]] - m) / denom;
    }
}

/* Dynamic-gating routing metadata (Sec. 5.1): the number of assignments of each
 * expert, their exclusive prefix sum (offsets[E] = k*T), and the sort index that
 * groups assignments by expert.  The sort is the stable one: inside an expert's
 * range rows are in ascending token order, so
 *   dst_row[t,j] = offsets[e] + #{t' < t : t' selected e},  e = idx[t,j],
 * and src_tok is its inverse (src_tok[dst_row[t,j]] = t).
 * Returns 0, or -1 if an index is outside [0,E). */
int moe_oracle_route(const int32_t *idx, int T, int E, int k,
                     int32_t *counts, int32_t *offsets, int32_t *dst_row, int32_t *src_tok)
{
    for (int e = 0; e < E; ++e)
        counts[e] = 0;
    for (size_t a = 0; a < (size_t)T * k; ++a) {
        if (idx[a] < 0 || idx[a] >= E)
            return -1;
        counts[idx[a]] += 1;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e)
        offsets[e + 1] = offsets[e] + counts[e];
    int32_t *seen = (int32_t *)calloc((size_t)E > 0 ? E : 1, sizeof(int32_t));
    for (int t = 0; t < T; ++t) {
        for (int j = 0; j < k; ++j) {
            int e = idx[(size_t)t * k + j];
            int r = offsets[e] + seen[e]; /* seen[e] = earlier tokens that chose e */
            dst_row[(size_t)t * k + j] = r;
            src_tok[r] = t;
        }
        for (int j = 0; j < k; ++j)
            seen[idx[(size_t)t * k + j]] += 1;
    }
    free(seen);
    return 0;
}

/* One expert FFN on one row (Sec. 2.2: the FFN block; ReLU as in the benchmark
 * definition):  out[d] = sum_f relu(sum_d' xin[d'] W1[e,f,d'] + b1[e,f]) * W2[e,d,f] + b2[e,d].
 * h is scratch of F doubles. */
static void ffn_row(const float *xin, int e, const void *w1, const void *w2,
                    const void *b1, const void *b2, int D, int F, int dt,
                    double *h, double *out)
{
    for (int f = 0; f < F; ++f) {
        size_t base = ((size_t)e * F + f) * D;
        double acc = dt == 0 ? dot_ff(xin, (const float *)w1 + base, D)
                             : dot_fb(xin, (const uint16_t *)w1 + base, D);
        if (b1)
            acc += ld(b1, (size_t)e * F + f, dt);
        h[f] = acc > 0.0 ? acc : 0.0;
    }
    for (int d = 0; d < D; ++d) {
        size_t base = ((size_t)e * D + d) * F;
        double acc = dt == 0 ? dot_df(h, (const float *)w2 + base, F)
                             : dot_db(h, (const uint16_t *)w2 + base, F);
        if (b2)
            acc += ld(b2, (size_t)e * D + d, dt);
        out[d] = acc;
    }
}

static void widen_row(const void *x, size_t row, int D, int dt, float *dst)
{
    for (int d = 0; d < D; ++d)
        dst[d] = (float)ld(x, row * D + d, dt);
}

/* Layer output for a list of tokens (all tokens when tokens == NULL, n = T):
 *   y[i,:] = sum_{j = 0..k-1, in this order} w[t,j] * FFN_{idx[t,j]}(x[t,:]),  t = tokens[i].
 * keep [T,k] (may be NULL) marks assignments that take part (1) or were dropped by a
 * static capacity (0).  Each output row depends only on its own token, so a sample
 * of tokens is exact.  y is fp64 [n,D]. */
void moe_oracle_layer_tokens(const void *x, const void *w1, const void *w2,
                             const void *b1, const void *b2,
                             const int32_t *idx, const double *w, const uint8_t *keep,
                             const int32_t *tokens, int n, int D, int F, int k, int dt,
                             double *y)
{
#pragma omp parallel
    {
        float *xin = (float *)malloc(sizeof(float) * (size_t)D);
        double *h = (double *)malloc(sizeof(double) * (size_t)F);
        double *o = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n; ++i) {
            int t = tokens ? tokens[i] : i;
            double *yr = y + (size_t)i * D;
            for (int d = 0; d < D; ++d)
                yr[d] = 0.0;
            widen_row(x, (size_t)t, D, dt, xin);
            for (int j = 0; j < k; ++j) {
                if (keep && !keep[(size_t)t * k + j])
                    continue;
                ffn_row(xin, idx[(size_t)t * k + j], w1, w2, b1, b2, D, F, dt, h, o);
                double g = w[(size_t)t * k + j];
                for (int d = 0; d < D; ++d)
                    yr[d] += g * o[d];
            }
        }
        free(xin);
        free(h);
        free(o);
    }
}

/* Grouped expert FFN on already dispatched rows: row r of xp belongs to the expert e
 * with offsets[e] <= r < offsets[e+1]; yp[r,:] = FFN_e(xp[r,:]).  rows == NULL means
 * all N rows, else only the listed ones (output row i for rows[i]).  yp fp64. */
void moe_oracle_expert_ffn_rows(const void *xp, const int32_t *offsets, int E,
                                const void *w1, const void *w2, const void *b1, const void *b2,
                                const int32_t *rows, int n, int D, int F, int dt, double *yp)
{
#pragma omp parallel
    {
        float *xin = (float *)malloc(sizeof(float) * (size_t)D);
        double *h = (double *)malloc(sizeof(double) * (size_t)F);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n; ++i) {
            int r = rows ? rows[i] : i;
            int e = 0;
            while (e < E && !(offsets[e] <= r && r < offsets[e + 1]))
                ++e;
            widen_row(xp, (size_t)r, D, dt, xin);
            ffn_row(xin, e, w1, w2, b1, b2, D, F, dt, h, yp + (size_t)i * D);
        }
        free(xin);
        free(h);
    }
}

/* Static gating bookkeeping (Sec. 3.2; Sec. 5.1, the dispatch-mask rule): every
 * expert owns `capacity` rows.  Assignments are visited slot by slot (all first
 * choices in token order, then all second choices, ...); an assignment takes the
 * first empty row of its expert, and is dropped when the expert is full.
 * slot[t,j] = row inside the expert (0..capacity-1) or -1 if dropped;
 * keep[t,j] = 1/0.  Returns the number of dropped assignments. */
int moe_oracle_static_slots(const int32_t *idx, int T, int E, int k, int capacity,
                            int32_t *slot, uint8_t *keep)
{
    int dropped = 0;
    int32_t *fill = (int32_t *)calloc((size_t)E > 0 ? E : 1, sizeof(int32_t));
    for (int j = 0; j < k; ++j) {
        for (int t = 0; t < T; ++t) {
            int e = idx[(size_t)t * k + j];
            if (fill[e] < capacity) {
                slot[(size_t)t * k + j] = fill[e];
                keep[(size_t)t * k + j] = 1;
                fill[e] += 1;
            } else {
                slot[(size_t)t * k + j] = -1;
                keep[(size_t)t * k + j] = 0;
                dropped += 1;
            }
        }
    }
    free(fill);
    return dropped;
}
