// Plain one-thread-per-output contractions for the replayed MoE layer.
// They serve the f32 activation dtype and any bf16 shape the MFMA kernels do not
// tile (hidden sizes that are not multiples of their tile edges).  f32
// accumulation in a fixed order; correctness first, speed is not a goal here.
#include "r3_kernels.h"

namespace r3 {

// expert that owns permuted row r: offsets[e] <= r < offsets[e+1]
__device__ __forceinline__ int expert_of_row(const int32_t *offsets, int E, int r) {
    int lo = 0, hi = E;  // invariant: offsets[lo] <= r < offsets[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (offsets[mid] <= r) lo = mid; else hi = mid;
    }
    return lo;
}

// s[t,e] = sum_c x[t,c] Wr[c,e] (+ bias[e])      (Section 4.1, router logits)
template <typename T>
__global__ void __launch_bounds__(256)
simt_logits_kernel(int Tn, int d, int E, const T *__restrict__ x, const T *__restrict__ Wr,
                   const float *__restrict__ bias, float *__restrict__ s) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)Tn * E) return;
    int t = (int)(i / E), e = (int)(i - (int64_t)t * E);
    float acc = 0.0f;
    for (int c = 0; c < d; ++c) acc = fmaf(Elem<T>::ld(x + (int64_t)t * d + c), Elem<T>::ld(Wr + (int64_t)c * E + e), acc);
    if (bias) acc += bias[e];
    s[i] = acc;
}

// A = Xp Wg[e], B = Xp Wu[e], H = silu(A) * B; saved for the backward: FA = B silu'(A), FB = silu(A)
template <typename T>
__global__ void __launch_bounds__(256)
simt_ffn1_kernel(int S, int d, int E, int F, const T *__restrict__ Xp, const int32_t *__restrict__ perm, int K,
                 const int32_t *__restrict__ offsets, const T *__restrict__ Wg, const T *__restrict__ Wu,
                 T *__restrict__ H, T *__restrict__ FA, T *__restrict__ FB, const float *__restrict__ grow) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)S * F) return;
    int r = (int)(i / F), f = (int)(i - (int64_t)r * F);
    int e = expert_of_row(offsets, E, r);
    const T *wg = Wg + (int64_t)e * d * F + f, *wu = Wu + (int64_t)e * d * F + f;
    const int src = perm ? perm[r] / K : r;   // perm given: Xp is x [T,d], row r reads its token
    float a = 0.0f, b = 0.0f;
    for (int c = 0; c < d; ++c) {
        float xv = Elem<T>::ld(Xp + (int64_t)src * d + c);
        a = fmaf(xv, Elem<T>::ld(wg + (int64_t)c * F), a);
        b = fmaf(xv, Elem<T>::ld(wu + (int64_t)c * F), b);
    }
    const float sg = sigmoidf_(a);
    Elem<T>::st(H + i, (grow ? grow[r] : 1.0f) * (a * sg * b));
    if (FA) Elem<T>::st(FA + i, b * sg * (1.0f + a * (1.0f - sg)));
    if (FB) Elem<T>::st(FB + i, a * sg);
}

// Yp = H Wd[e]
template <typename T>
__global__ void __launch_bounds__(256)
simt_ffn2_kernel(int S, int d, int E, int F, const T *__restrict__ H, const int32_t *__restrict__ offsets,
                 const T *__restrict__ Wd, T *__restrict__ Yp) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)S * d) return;
    int r = (int)(i / d), c = (int)(i - (int64_t)r * d);
    int e = expert_of_row(offsets, E, r);
    const T *wd = Wd + (int64_t)e * F * d + c;
    float acc = 0.0f;
    for (int f = 0; f < F; ++f) acc = fmaf(Elem<T>::ld(H + (int64_t)r * F + f), Elem<T>::ld(wd + (int64_t)f * d), acc);
    Elem<T>::st(Yp + i, acc);
}

// dh = dYp Wd[e]^T ; dA = dh * FA ; dB = dh * FB   (FA = B silu'(A), FB = silu(A) from the forward)
template <typename T>
__global__ void __launch_bounds__(256)
simt_dh_kernel(int S, int d, int E, int F, const T *__restrict__ dYp, const int32_t *__restrict__ offsets,
               const T *__restrict__ Wd, const T *__restrict__ FA, const T *__restrict__ FB,
               T *__restrict__ dA, T *__restrict__ dB) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)S * F) return;
    int r = (int)(i / F), f = (int)(i - (int64_t)r * F);
    int e = expert_of_row(offsets, E, r);
    const T *wd = Wd + ((int64_t)e * F + f) * d;
    float dh = 0.0f;
    for (int c = 0; c < d; ++c) dh = fmaf(Elem<T>::ld(dYp + (int64_t)r * d + c), Elem<T>::ld(wd + c), dh);
    Elem<T>::st(dA + i, dh * Elem<T>::ld(FA + i));
    Elem<T>::st(dB + i, dh * Elem<T>::ld(FB + i));
}

// dXp = dA Wg[e]^T + dB Wu[e]^T
template <typename T>
__global__ void __launch_bounds__(256)
simt_dxp_kernel(int S, int d, int E, int F, const T *__restrict__ dA, const T *__restrict__ dB,
                const int32_t *__restrict__ offsets, const T *__restrict__ Wg, const T *__restrict__ Wu,
                T *__restrict__ dXp) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)S * d) return;
    int r = (int)(i / d), c = (int)(i - (int64_t)r * d);
    int e = expert_of_row(offsets, E, r);
    const T *wg = Wg + ((int64_t)e * d + c) * F, *wu = Wu + ((int64_t)e * d + c) * F;
    float acc = 0.0f;
    for (int f = 0; f < F; ++f) acc = fmaf(Elem<T>::ld(dA + (int64_t)r * F + f), Elem<T>::ld(wg + f), acc);
    for (int f = 0; f < F; ++f) acc = fmaf(Elem<T>::ld(dB + (int64_t)r * F + f), Elem<T>::ld(wu + f), acc);
    Elem<T>::st(dXp + i, acc);
}

// out[e][p][q] (+)= sum_{r in expert e} P[r][p] * Q[r][q]   (weight gradients)
// ptok / qtok != NULL: that operand is an un-permuted matrix and row r of the reduction is its row tok[r]
template <typename T>
__global__ void __launch_bounds__(256)
simt_wgrad_kernel(int E, int NP, int NQ, const T *__restrict__ P, const int32_t *__restrict__ ptok,
                  const T *__restrict__ Q, const int32_t *__restrict__ qtok, const int32_t *__restrict__ offsets,
                  float *__restrict__ out, int accumulate) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)E * NP * NQ) return;
    int e = (int)(i / ((int64_t)NP * NQ));
    int64_t rem = i - (int64_t)e * NP * NQ;
    int p = (int)(rem / NQ), q = (int)(rem - (int64_t)p * NQ);
    float acc = 0.0f;
    for (int r = offsets[e]; r < offsets[e + 1]; ++r)
        acc = fmaf(Elem<T>::ld(P + (int64_t)(ptok ? ptok[r] : r) * NP + p),
                   Elem<T>::ld(Q + (int64_t)(qtok ? qtok[r] : r) * NQ + q), acc);
    out[i] = accumulate ? out[i] + acc : acc;
}

// dWr[c][e] (+)= sum_t x[t][c] ds[t][e]
template <typename T>
__global__ void __launch_bounds__(256)
simt_dwr_kernel(int Tn, int d, int E, const T *__restrict__ x, const T *__restrict__ ds,
                float *__restrict__ dWr, int accumulate) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)d * E) return;
    int c = (int)(i / E), e = (int)(i - (int64_t)c * E);
    const int dsw = (sizeof(T) == 2) ? 2 * E : E;  // bf16: ds rows are [hi(E) | lo(E)]
    float acc = 0.0f;
    for (int t = 0; t < Tn; ++t) {
        float dv = Elem<T>::ld(ds + (int64_t)t * dsw + e);
        if (sizeof(T) == 2) dv += Elem<T>::ld(ds + (int64_t)t * dsw + E + e);
        acc = fmaf(Elem<T>::ld(x + (int64_t)t * d + c), dv, acc);
    }
    dWr[i] = accumulate ? dWr[i] + acc : acc;
}

static inline int blocks_for(int64_t n) { return (int)((n + 255) / 256); }

#define R3_BY_ACT(act, CALL_BF16, CALL_F32) \
    do { if ((act) == R3_BF16) { CALL_BF16; } else { CALL_F32; } } while (0)

hipError_t simt_router_logits(int T, int d, int E, int act, const void *x, const void *Wr, const float *bias,
                              float *logits, hipStream_t s) {
    int g = blocks_for((int64_t)T * E);
    R3_BY_ACT(act, (simt_logits_kernel<bf16_t><<<g, 256, 0, s>>>(T, d, E, (const bf16_t *)x, (const bf16_t *)Wr, bias, logits)),
              (simt_logits_kernel<float><<<g, 256, 0, s>>>(T, d, E, (const float *)x, (const float *)Wr, bias, logits)));
    return hipGetLastError();
}

hipError_t simt_ffn1(int S, int d, int E, int F, int act, const void *Xp, const int32_t *perm, int K,
                     const int32_t *offsets, const void *Wg, const void *Wu, void *H, void *A, void *B,
                     const float *grow, hipStream_t s) {
    int g = blocks_for((int64_t)S * F);
    R3_BY_ACT(act, (simt_ffn1_kernel<bf16_t><<<g, 256, 0, s>>>(S, d, E, F, (const bf16_t *)Xp, perm, K, offsets, (const bf16_t *)Wg, (const bf16_t *)Wu, (bf16_t *)H, (bf16_t *)A, (bf16_t *)B, grow)),
              (simt_ffn1_kernel<float><<<g, 256, 0, s>>>(S, d, E, F, (const float *)Xp, perm, K, offsets, (const float *)Wg, (const float *)Wu, (float *)H, (float *)A, (float *)B, grow)));
    return hipGetLastError();
}

hipError_t simt_ffn2(int S, int d, int E, int F, int act, const void *H, const int32_t *offsets, const void *Wd,
                     void *Yp, hipStream_t s) {
    int g = blocks_for((int64_t)S * d);
    R3_BY_ACT(act, (simt_ffn2_kernel<bf16_t><<<g, 256, 0, s>>>(S, d, E, F, (const bf16_t *)H, offsets, (const bf16_t *)Wd, (bf16_t *)Yp)),
              (simt_ffn2_kernel<float><<<g, 256, 0, s>>>(S, d, E, F, (const float *)H, offsets, (const float *)Wd, (float *)Yp)));
    return hipGetLastError();
}

hipError_t simt_dh(int S, int d, int E, int F, int act, const void *dYp, const int32_t *offsets, const void *Wd,
                   const void *A, const void *B, void *dA, void *dB, hipStream_t s) {
    int g = blocks_for((int64_t)S * F);
    R3_BY_ACT(act, (simt_dh_kernel<bf16_t><<<g, 256, 0, s>>>(S, d, E, F, (const bf16_t *)dYp, offsets, (const bf16_t *)Wd, (const bf16_t *)A, (const bf16_t *)B, (bf16_t *)dA, (bf16_t *)dB)),
              (simt_dh_kernel<float><<<g, 256, 0, s>>>(S, d, E, F, (const float *)dYp, offsets, (const float *)Wd, (const float *)A, (const float *)B, (float *)dA, (float *)dB)));
    return hipGetLastError();
}

hipError_t simt_dxp(int S, int d, int E, int F, int act, const void *dA, const void *dB, const int32_t *offsets,
                    const void *Wg, const void *Wu, void *dXp, hipStream_t s) {
    int g = blocks_for((int64_t)S * d);
    R3_BY_ACT(act, (simt_dxp_kernel<bf16_t><<<g, 256, 0, s>>>(S, d, E, F, (const bf16_t *)dA, (const bf16_t *)dB, offsets, (const bf16_t *)Wg, (const bf16_t *)Wu, (bf16_t *)dXp)),
              (simt_dxp_kernel<float><<<g, 256, 0, s>>>(S, d, E, F, (const float *)dA, (const float *)dB, offsets, (const float *)Wg, (const float *)Wu, (float *)dXp)));
    return hipGetLastError();
}

hipError_t simt_wgrad(int E, int NP, int NQ, int act, const void *P, const int32_t *ptok, const void *Q,
                      const int32_t *qtok, const int32_t *offsets, float *out, int accumulate, hipStream_t s) {
    int g = blocks_for((int64_t)E * NP * NQ);
    R3_BY_ACT(act, (simt_wgrad_kernel<bf16_t><<<g, 256, 0, s>>>(E, NP, NQ, (const bf16_t *)P, ptok, (const bf16_t *)Q, qtok, offsets, out, accumulate)),
              (simt_wgrad_kernel<float><<<g, 256, 0, s>>>(E, NP, NQ, (const float *)P, ptok, (const float *)Q, qtok, offsets, out, accumulate)));
    return hipGetLastError();
}

hipError_t simt_dwr(int T, int d, int E, int act, const void *x, const void *ds, float *dWr, int accumulate,
                    hipStream_t s) {
    int g = blocks_for((int64_t)d * E);
    R3_BY_ACT(act, (simt_dwr_kernel<bf16_t><<<g, 256, 0, s>>>(T, d, E, (const bf16_t *)x, (const bf16_t *)ds, dWr, accumulate)),
              (simt_dwr_kernel<float><<<g, 256, 0, s>>>(T, d, E, (const float *)x, (const float *)ds, dWr, accumulate)));
    return hipGetLastError();
}

}  // namespace r3
