/*
 * CPU oracle for the replayed-routing MoE layer of Rollout Routing Replay
 * (arxiv 2510.11370, Section 4.1 "Implementation").
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision
 * restatement of the layer's definition and is only ever called from the
 * tests, from the smoke check and from the benchmark's cpu_baseline leg.
 * The GPU library never calls it and shares no code with it.
 *
 * Notation follows the paper: E experts (the paper's M), K selected experts,
 * T tokens, d hidden size, F expert width.  A "slot" is one (token t, j) pair,
 * slot id = t*K + j.  Every function takes host pointers.  Floating-point
 * inputs arrive as float (bf16-rounded values are exact in float) and are
 * widened to double; nothing is rounded in between; outputs are double.
 *
 * What the paper leaves open and the reading taken here:
 *   - expert network E_i: bias-free SwiGLU, W_down(silu(x W_gate) * (x W_up));
 *   - TopKMask ties: lower expert id wins; NaN ranks below every number;
 *     -0 equals +0; the K indices of a token are stored ascending by id;
 *   - dispatch order: stable, i.e. rows of one expert keep ascending slot id;
 *   - backward: derivative of sum(dy*y) with the recorded mask held constant.
 *
 * All functions are pinned by tests/test_oracle_*.py (none is parity-unpinned).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- Section 4.1, first equation: router logits  s = x W_r (+ bias) ------- */
/* x [T,d], Wr [d,E] row-major, bias [E] or NULL, s [T,E]. */
void oracle_router_logits(int T, int d, int E, const float *x, const float *Wr,
                          const float *bias, double *s)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double *row = s + (size_t)t * E;
        for (int e = 0; e < E; ++e)
            row[e] = 0.0;
        for (int c = 0; c < d; ++c) {
            double xv = (double)x[(size_t)t * d + c];
            const float *w = Wr + (size_t)c * E;
            for (int e = 0; e < E; ++e)
                row[e] += xv * (double)w[e];
        }
        if (bias)
            for (int e = 0; e < E; ++e)
                row[e] += (double)bias[e];
    }
}

/* "a ranks strictly ahead of b" in the order used for TopKMask:
 * larger value first, equal values by lower expert id, NaN after everything. */
static int ranks_ahead(double va, int ia, double vb, int ib)
{
    int na = isnan(va), nb = isnan(vb);
    if (na || nb) {
        if (na && nb)
            return ia < ib;
        return nb; /* a number beats a NaN */
    }
    if (va > vb)
        return 1;
    if (va < vb)
        return 0;
    return ia < ib; /* equal (this also makes -0 == +0) */
}

/* ---- Section 4.1, TopKMask(s, K): the mask as K expert ids ---------------- */
/* logits [T,E] double; idx [T,K] int32, ascending inside a token.
 * An expert is selected when fewer than K experts rank ahead of it. */
void oracle_topk_mask_f64(int T, int E, int K, const double *logits, int32_t *idx)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const double *row = logits + (size_t)t * E;
        int n = 0;
        for (int e = 0; e < E; ++e) {
            int ahead = 0;
            for (int f = 0; f < E; ++f)
                if (f != e && ranks_ahead(row[f], f, row[e], e))
                    ++ahead;
            if (ahead < K)
                idx[(size_t)t * K + n++] = e; /* e ascends, so the ids do */
        }
    }
}

/* Same, for the float logits buffer the inference side hands over. */
void oracle_topk_mask_f32(int T, int E, int K, const float *logits, int32_t *idx)
{
    double *tmp = (double *)malloc((size_t)T * E * sizeof(double));
    for (size_t i = 0; i < (size_t)T * E; ++i)
        tmp[i] = (double)logits[i];
    oracle_topk_mask_f64(T, E, K, tmp, idx);
    free(tmp);
}

/* ---- Section 4.1, replay gate: softmax of the training logits over the
 *      recorded expert set ------------------------------------------------- */
/* s [T,E] training logits, idx [T,K] recorded ids, g [T,K] aligned with idx.
 * Subtracting the row maximum changes nothing mathematically. */
void oracle_replay_gate(int T, int E, int K, const double *s, const int32_t *idx,
                        double *g)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const double *row = s + (size_t)t * E;
        const int32_t *id = idx + (size_t)t * K;
        double *gt = g + (size_t)t * K;
        double m = row[id[0]];
        for (int j = 1; j < K; ++j)
            if (row[id[j]] > m)
                m = row[id[j]];
        double den = 0.0;
        for (int j = 0; j < K; ++j) {
            gt[j] = exp(row[id[j]] - m);
            den += gt[j];
        }
        for (int j = 0; j < K; ++j)
            gt[j] /= den;
    }
}

/* ---- dispatch implied by the output equation: sort slots by expert -------- */
/* counts [E], offsets [E+1], inv_perm [T*K] (slot -> row), perm [T*K] (row -> slot). */
void oracle_permute(int T, int E, int K, const int32_t *idx, int32_t *counts,
                    int32_t *offsets, int32_t *inv_perm, int32_t *perm)
{
    size_t S = (size_t)T * K;
    for (int e = 0; e < E; ++e)
        counts[e] = 0;
    for (size_t sl = 0; sl < S; ++sl)
        counts[idx[sl]]++;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e)
        offsets[e + 1] = offsets[e] + counts[e];
    int32_t *fill = (int32_t *)calloc(E > 0 ? (size_t)E : 1u, sizeof(int32_t));
    for (size_t sl = 0; sl < S; ++sl) {
        int e = idx[sl];
        int32_t row = offsets[e] + fill[e]++;
        inv_perm[sl] = row;
        perm[row] = (int32_t)sl;
    }
    free(fill);
}

/* Xp[row] = x[perm[row] / K]  (rows are copies). */
void oracle_gather_rows(int T, int K, int d, const float *x, const int32_t *perm,
                        float *Xp)
{
    size_t S = (size_t)T * K;
    for (size_t r = 0; r < S; ++r)
        memcpy(Xp + r * d, x + (size_t)(perm[r] / K) * d, (size_t)d * sizeof(float));
}

static double sigmoid(double v) { return 1.0 / (1.0 + exp(-v)); }

/* ---- expert network E_i of the output equation, as SwiGLU, for the rows
 *      [r0, r1) that belong to one expert ---------------------------------- */
/* Xp [*,d] float; Wg, Wu [d,F]; Wd [F,d] (this expert's matrices);
 * a, b, h [*,F] and o [*,d] double, addressed by absolute row. */
static void expert_rows(int r0, int r1, int d, int F, const float *Xp,
                        const float *Wg, const float *Wu, const float *Wd,
                        double *a, double *b, double *h, double *o)
{
#pragma omp parallel for schedule(static)
    for (int r = r0; r < r1; ++r) {
        const float *xr = Xp + (size_t)r * d;
        double *ar = a + (size_t)r * F, *br = b + (size_t)r * F;
        double *hr = h + (size_t)r * F, *orow = o + (size_t)r * d;
        for (int f = 0; f < F; ++f)
            ar[f] = br[f] = 0.0;
        for (int c = 0; c < d; ++c) {
            double xv = (double)xr[c];
            const float *wg = Wg + (size_t)c * F, *wu = Wu + (size_t)c * F;
            for (int f = 0; f < F; ++f) {
                ar[f] += xv * (double)wg[f];
                br[f] += xv * (double)wu[f];
            }
        }
        for (int f = 0; f < F; ++f)
            hr[f] = ar[f] * sigmoid(ar[f]) * br[f];
        for (int c = 0; c < d; ++c)
            orow[c] = 0.0;
        for (int f = 0; f < F; ++f) {
            double hv = hr[f];
            const float *wd = Wd + (size_t)f * d;
            for (int c = 0; c < d; ++c)
                orow[c] += hv * (double)wd[c];
        }
    }
}

/* Grouped form: expert e owns rows offsets[e] .. offsets[e+1].
 * Wg, Wu [E,d,F]; Wd [E,F,d]. */
void oracle_grouped_ffn(int E, int d, int F, const int32_t *offsets, const float *Xp,
                        const float *Wg, const float *Wu, const float *Wd,
                        double *a, double *b, double *h, double *o)
{
    for (int e = 0; e < E; ++e)
        expert_rows(offsets[e], offsets[e + 1], d, F, Xp,
                    Wg + (size_t)e * d * F, Wu + (size_t)e * d * F,
                    Wd + (size_t)e * F * d, a, b, h, o);
}

/* ---- Section 4.1, replay output: y_t = sum_j g[t,j] * o[row of slot (t,j)] - */
void oracle_combine(int T, int K, int d, const double *o, const double *g,
                    const int32_t *inv_perm, double *y)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double *yt = y + (size_t)t * d;
        for (int c = 0; c < d; ++c)
            yt[c] = 0.0;
        for (int j = 0; j < K; ++j) {
            double gj = g[(size_t)t * K + j];
            const double *orow = o + (size_t)inv_perm[(size_t)t * K + j] * d;
            for (int c = 0; c < d; ++c)
                yt[c] += gj * orow[c];
        }
    }
}

/* ---- the whole forward, steps in the order of Section 4.1 ----------------- */
/* Outputs that the backward needs are returned too.  Buffers are the caller's:
 * s [T,E], g [T,K], counts [E], offsets [E+1], inv_perm/perm [T*K],
 * Xp [T*K,d] float, a/b/h [T*K,F], o [T*K,d], y [T,d]. */
void oracle_moe_forward(int T, int d, int E, int K, int F, const float *x,
                        const float *Wr, const float *bias, const int32_t *idx,
                        const float *Wg, const float *Wu, const float *Wd,
                        double *s, double *g, int32_t *counts, int32_t *offsets,
                        int32_t *inv_perm, int32_t *perm, float *Xp, double *a,
                        double *b, double *h, double *o, double *y)
{
    oracle_router_logits(T, d, E, x, Wr, bias, s);
    oracle_replay_gate(T, E, K, s, idx, g);
    oracle_permute(T, E, K, idx, counts, offsets, inv_perm, perm);
    oracle_gather_rows(T, K, d, x, perm, Xp);
    oracle_grouped_ffn(E, d, F, offsets, Xp, Wg, Wu, Wd, a, b, h, o);
    oracle_combine(T, K, d, o, g, inv_perm, y);
}

/* ---- backward of the replayed layer (the paper only states that gradients
 *      reach the logits through the softmax; this is that derivative, the
 *      recorded mask being a constant) -------------------------------------- */

/* Through the combine and the masked softmax.
 * dg_j = <dy_t, o_j>, do_j = g_j dy_t, dz_j = g_j (dg_j - sum_i g_i dg_i).
 * dz [T,K] aligned with idx; ds [T,E] dense, zero off the recorded set;
 * dO [T*K,d] by row. */
void oracle_gate_backward(int T, int d, int E, int K, const float *dy,
                          const double *o, const double *g, const int32_t *idx,
                          const int32_t *inv_perm, double *dO, double *dz, double *ds)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *dyt = dy + (size_t)t * d;
        double *dzt = dz + (size_t)t * K;
        double mix = 0.0;
        for (int j = 0; j < K; ++j) {
            size_t row = (size_t)inv_perm[(size_t)t * K + j];
            double gj = g[(size_t)t * K + j], dot = 0.0;
            for (int c = 0; c < d; ++c) {
                dot += (double)dyt[c] * o[row * d + c];
                dO[row * d + c] = gj * (double)dyt[c];
            }
            dzt[j] = dot; /* dg_j for now */
            mix += gj * dot;
        }
        for (int e = 0; e < E; ++e)
            ds[(size_t)t * E + e] = 0.0;
        for (int j = 0; j < K; ++j) {
            dzt[j] = g[(size_t)t * K + j] * (dzt[j] - mix);
            ds[(size_t)t * E + idx[(size_t)t * K + j]] = dzt[j];
        }
    }
}

/* Router: dWr = x^T ds, dbias = column sums of ds, dx_router = ds Wr^T.
 * dWr [d,E], dbias [E] (may be NULL), dxr [T,d]. */
void oracle_router_backward(int T, int d, int E, const float *x, const float *Wr,
                            const double *ds, double *dWr, double *dbias, double *dxr)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < d; ++c) {
        double *w = dWr + (size_t)c * E;
        for (int e = 0; e < E; ++e)
            w[e] = 0.0;
        for (int t = 0; t < T; ++t) { /* tokens in ascending order */
            double xv = (double)x[(size_t)t * d + c];
            for (int e = 0; e < E; ++e)
                w[e] += xv * ds[(size_t)t * E + e];
        }
    }
    if (dbias)
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int t = 0; t < T; ++t)
                acc += ds[(size_t)t * E + e];
            dbias[e] = acc;
        }
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int e = 0; e < E; ++e)
                acc += ds[(size_t)t * E + e] * (double)Wr[(size_t)c * E + e];
            dxr[(size_t)t * d + c] = acc;
        }
}

/* One expert's rows [r0, r1): dh = do Wd^T; da = dh * b * silu'(a);
 * db = dh * silu(a); dWd = h^T do; dWg = Xp^T da; dWu = Xp^T db;
 * dXp = da Wg^T + db Wu^T.  da/db [*,F] and dXp [*,d] by absolute row;
 * dWg, dWu [d,F] and dWd [F,d] are this expert's (overwritten). */
static void expert_rows_backward(int r0, int r1, int d, int F, const float *Xp,
                                 const float *Wg, const float *Wu, const float *Wd,
                                 const double *a, const double *b, const double *h,
                                 const double *dO, double *da, double *db,
                                 double *dXp, double *dWg, double *dWu, double *dWd)
{
#pragma omp parallel for schedule(static)
    for (int r = r0; r < r1; ++r) {
        const double *dor = dO + (size_t)r * d;
        for (int f = 0; f < F; ++f) {
            const float *wd = Wd + (size_t)f * d;
            double dh = 0.0;
            for (int c = 0; c < d; ++c)
                dh += dor[c] * (double)wd[c];
            double av = a[(size_t)r * F + f], bv = b[(size_t)r * F + f];
            double sg = sigmoid(av);
            da[(size_t)r * F + f] = dh * bv * sg * (1.0 + av * (1.0 - sg));
            db[(size_t)r * F + f] = dh * av * sg;
        }
        const double *dar = da + (size_t)r * F, *dbr = db + (size_t)r * F;
        for (int c = 0; c < d; ++c) {
            const float *wg = Wg + (size_t)c * F, *wu = Wu + (size_t)c * F;
            double acc = 0.0;
            for (int f = 0; f < F; ++f)
                acc += dar[f] * (double)wg[f] + dbr[f] * (double)wu[f];
            dXp[(size_t)r * d + c] = acc;
        }
    }
#pragma omp parallel for schedule(static)
    for (int f = 0; f < F; ++f) {
        double *w = dWd + (size_t)f * d;
        for (int c = 0; c < d; ++c)
            w[c] = 0.0;
        for (int r = r0; r < r1; ++r) { /* rows in ascending order */
            double hv = h[(size_t)r * F + f];
            for (int c = 0; c < d; ++c)
                w[c] += hv * dO[(size_t)r * d + c];
        }
    }
#pragma omp parallel for schedule(static)
    for (int c = 0; c < d; ++c) {
        double *wg = dWg + (size_t)c * F, *wu = dWu + (size_t)c * F;
        for (int f = 0; f < F; ++f)
            wg[f] = wu[f] = 0.0;
        for (int r = r0; r < r1; ++r) {
            double xv = (double)Xp[(size_t)r * d + c];
            for (int f = 0; f < F; ++f) {
                wg[f] += xv * da[(size_t)r * F + f];
                wu[f] += xv * db[(size_t)r * F + f];
            }
        }
    }
}

void oracle_grouped_ffn_backward(int E, int d, int F, const int32_t *offsets,
                                 const float *Xp, const float *Wg, const float *Wu,
                                 const float *Wd, const double *a, const double *b,
                                 const double *h, const double *dO, double *da,
                                 double *db, double *dXp, double *dWg, double *dWu,
                                 double *dWd)
{
    for (int e = 0; e < E; ++e)
        expert_rows_backward(offsets[e], offsets[e + 1], d, F, Xp,
                             Wg + (size_t)e * d * F, Wu + (size_t)e * d * F,
                             Wd + (size_t)e * F * d, a, b, h, dO, da, db, dXp,
                             dWg + (size_t)e * d * F, dWu + (size_t)e * d * F,
                             dWd + (size_t)e * F * d);
}

/* dx_t = dx_router_t + sum_j dXp[row of slot (t,j)]. */
void oracle_unpermute_add(int T, int K, int d, const double *dxr, const double *dXp,
                          const int32_t *inv_perm, double *dx)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int c = 0; c < d; ++c) {
            double acc = dxr[(size_t)t * d + c];
            for (int j = 0; j < K; ++j)
                acc += dXp[(size_t)inv_perm[(size_t)t * K + j] * d + c];
            dx[(size_t)t * d + c] = acc;
        }
}

/* Whole backward from the forward's saved values.  Scratch (caller's):
 * dO [T*K,d], dz [T,K], ds [T,E], dxr [T,d], da/db [T*K,F], dXp [T*K,d]. */
void oracle_moe_backward(int T, int d, int E, int K, int F, const float *dy,
                         const float *x, const float *Wr, const int32_t *idx,
                         const float *Wg, const float *Wu, const float *Wd,
                         const double *g, const int32_t *offsets,
                         const int32_t *inv_perm, const float *Xp, const double *a,
                         const double *b, const double *h, const double *o,
                         double *dO, double *dz, double *ds, double *dxr, double *da,
                         double *db, double *dXp, double *dx, double *dWr,
                         double *dbias, double *dWg, double *dWu, double *dWd)
{
    oracle_gate_backward(T, d, E, K, dy, o, g, idx, inv_perm, dO, dz, ds);
    oracle_router_backward(T, d, E, x, Wr, ds, dWr, dbias, dxr);
    oracle_grouped_ffn_backward(E, d, F, offsets, Xp, Wg, Wu, Wd, a, b, h, dO, da, db,
                                dXp, dWg, dWu, dWd);
    oracle_unpermute_add(T, K, d, dxr, dXp, inv_perm, dx);
}

/* ---- routing agreement between two records (Section 3.2, router level) ---- */
/* out[0] = tokens whose two expert sets are equal, out[1] = total number of
 * experts the two sets share (sum over tokens of |A and B|). */
void oracle_agreement(int T, int K, const int32_t *idx_a, const int32_t *idx_b,
                      int64_t *out)
{
    int64_t same = 0, shared = 0;
    for (int t = 0; t < T; ++t) {
        int n = 0;
        for (int i = 0; i < K; ++i)
            for (int j = 0; j < K; ++j)
                if (idx_a[(size_t)t * K + i] == idx_b[(size_t)t * K + j])
                    ++n;
        shared += n;
        if (n == K)
            ++same;
    }
    out[0] = same;
    out[1] = shared;
}

/* Number of threads the parallel loops above use (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) { omp_set_num_threads(n); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
