/* Drives every entry point of oracle/r3_oracle.c once on a tiny layer, with every buffer allocated at its
 * exact size, so that a build with -fsanitize=address,undefined reports any access outside a buffer, any
 * misaligned or overflowing arithmetic.  Test infrastructure (tests/test_oracle_sanitizers.py builds and
 * runs it on the CPU); prints "ok <checksum>". */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_topk_mask_f32(int T, int E, int K, const float *logits, int32_t *idx);
void oracle_topk_mask_f64(int T, int E, int K, const double *logits, int32_t *idx);
void oracle_moe_forward(int T, int d, int E, int K, int F, const float *x, const float *Wr, const float *bias,
                        const int32_t *idx, const float *Wg, const float *Wu, const float *Wd, double *s, double *g,
                        int32_t *counts, int32_t *offsets, int32_t *inv_perm, int32_t *perm, float *Xp, double *a,
                        double *b, double *h, double *o, double *y);
void oracle_moe_backward(int T, int d, int E, int K, int F, const float *dy, const float *x, const float *Wr,
                         const int32_t *idx, const float *Wg, const float *Wu, const float *Wd, const double *g,
                         const int32_t *offsets, const int32_t *inv_perm, const float *Xp, const double *a,
                         const double *b, const double *h, const double *o, double *dO, double *dz, double *ds,
                         double *dxr, double *da, double *db, double *dXp, double *dx, double *dWr, double *dbias,
                         double *dWg, double *dWu, double *dWd);
void oracle_agreement(int T, int K, const int32_t *idx_a, const int32_t *idx_b, int64_t *out);

static uint32_t rng = 12345u;
static float rnd(void) {   /* uniform in (-1, 1) */
    rng = rng * 1664525u + 1013904223u;
    return (float)((rng >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static float *fbuf(size_t n, float scale) {
    float *p = malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = scale * rnd();
    return p;
}
static double *dbuf(size_t n) { return malloc(n * sizeof(double)); }
static int32_t *ibuf(size_t n) { return malloc(n * sizeof(int32_t)); }

int main(void) {
    /* E = 7 with K = 2 of T = 9 tokens: some experts stay empty; odd sizes everywhere */
    enum { T = 9, d = 10, E = 7, K = 2, F = 6, S = T * K };
    float *x = fbuf(T * d, 1.0f), *Wr = fbuf(d * E, 0.3f), *bias = fbuf(E, 0.5f), *dy = fbuf(T * d, 1.0f);
    float *Wg = fbuf(E * d * F, 0.3f), *Wu = fbuf(E * d * F, 0.3f), *Wd = fbuf(E * F * d, 0.3f);
    float *lg = fbuf(T * E, 1.0f);
    lg[3] = lg[4];                    /* a tie */
    lg[E + 2] = NAN;                  /* a NaN ranks last */
    double *lg64 = dbuf(T * E);
    for (int i = 0; i < T * E; ++i) lg64[i] = lg[i];
    int32_t *idx = ibuf(S), *idx64 = ibuf(S);
    oracle_topk_mask_f32(T, E, K, lg, idx);
    oracle_topk_mask_f64(T, E, K, lg64, idx64);
    int64_t agree[2];
    oracle_agreement(T, K, idx, idx64, agree);
    if (agree[0] != T || agree[1] != S) { printf("top-K of the same values differs between f32 and f64\n"); return 1; }
    double *s = dbuf(T * E), *g = dbuf(T * K), *a = dbuf(S * F), *b = dbuf(S * F), *h = dbuf(S * F), *o = dbuf(S * d),
           *y = dbuf(T * d);
    int32_t *counts = ibuf(E), *offsets = ibuf(E + 1), *inv_perm = ibuf(S), *perm = ibuf(S);
    float *Xp = malloc(S * d * sizeof(float));
    oracle_moe_forward(T, d, E, K, F, x, Wr, bias, idx, Wg, Wu, Wd, s, g, counts, offsets, inv_perm, perm, Xp, a, b,
                       h, o, y);
    double *dO = dbuf(S * d), *dz = dbuf(T * K), *ds = dbuf(T * E), *dxr = dbuf(T * d), *da = dbuf(S * F),
           *db = dbuf(S * F), *dXp = dbuf(S * d), *dx = dbuf(T * d), *dWr = dbuf(d * E), *dbias = dbuf(E),
           *dWg = dbuf(E * d * F), *dWu = dbuf(E * d * F), *dWd = dbuf(E * F * d);
    oracle_moe_backward(T, d, E, K, F, dy, x, Wr, idx, Wg, Wu, Wd, g, offsets, inv_perm, Xp, a, b, h, o, dO, dz, ds,
                        dxr, da, db, dXp, dx, dWr, dbias, dWg, dWu, dWd);
    double sum = 0.0;
    for (int i = 0; i < T * d; ++i) sum += y[i] + dx[i];
    for (int i = 0; i < d * E; ++i) sum += dWr[i];
    for (int i = 0; i < E * d * F; ++i) sum += dWg[i] + dWu[i] + dWd[i];
    for (int i = 0; i < E; ++i) sum += dbias[i];
    if (offsets[E] != S || !isfinite(sum)) { printf("bad result\n"); return 1; }
    printf("ok %.6f\n", sum);
    return 0;
}
