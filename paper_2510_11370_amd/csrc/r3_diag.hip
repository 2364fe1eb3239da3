// Discrepancy diagnostics of Section 3 of arxiv 2510.11370 as HBM-bound reductions:
//   routing differences between two records (Section 3.2: router, token and sequence level),
//   k3 estimate of KL(pi_train || pi_infer) and the extreme-token fraction F(tau) (Section 3.1).
// Counts are integers (atomics on integers commute, so every result is reproducible); the one
// floating-point sum is reduced in a fixed order through per-block partials.
#include <cmath>

#include "r3_kernels.h"

namespace r3 {
namespace {

constexpr int kMaxTau = 8;
constexpr int kDiagBlocks = 1024;

// number of ids of a[0..K) that do not occur in b[0..K) (sets of distinct ids, any order)
template <typename IdxT>
__device__ __forceinline__ int differing(const IdxT *a, const IdxT *b, int K) {
    int common = 0;
    for (int i = 0; i < K; ++i) {
        const IdxT v = a[i];
        bool hit = false;
        for (int j = 0; j < K; ++j) hit |= (b[j] == v);
        common += hit;
    }
    return K - common;
}

// K = 8 one-byte ids: a router's set is one 64-bit word; equal words (the common case, the
// canonical ascending encoding) need no search, otherwise each byte of a is looked up in b
// with the zero-byte test on b ^ (byte replicated)
__device__ __forceinline__ int differing8(uint64_t a, uint64_t b) {
    if (a == b) return 0;
    int common = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint64_t rep = ((a >> (8 * i)) & 0xffull) * 0x0101010101010101ull;
        const uint64_t x = b ^ rep;
        common += ((x - 0x0101010101010101ull) & ~x & 0x8080808080808080ull) != 0ull;
    }
    return 8 - common;
}

// One thread per token, layers in a loop.  Layer-major records give coalesced 8-byte reads across
// the wave; token-major ones keep a thread on its own L*K bytes.
template <typename IdxT>
__global__ void __launch_bounds__(256)
routing_diff_kernel(int T, int K, int L, const IdxT *__restrict__ a, const IdxT *__restrict__ b,
                    int64_t token_stride, int64_t layer_stride, unsigned long long *__restrict__ router_hist,
                    int32_t *__restrict__ token_choices, int32_t *__restrict__ token_routers) {
    __shared__ int hist[kMaxK + 1];
    for (int i = threadIdx.x; i <= K; i += blockDim.x) hist[i] = 0;
    __syncthreads();
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) {
        int choices = 0, routers = 0;
        const bool words = sizeof(IdxT) == 1 && K == 8 && (token_stride % 8) == 0 && (layer_stride % 8) == 0 &&
                           ((uintptr_t)a % 8) == 0 && ((uintptr_t)b % 8) == 0;
        for (int l = 0; l < L; ++l) {
            const int64_t o = (int64_t)l * layer_stride + (int64_t)t * token_stride;
            const int d = words ? differing8(*(const uint64_t *)(a + o), *(const uint64_t *)(b + o))
                                : differing(a + o, b + o, K);
            choices += d;
            routers += d > 0;
            atomicAdd(&hist[d], 1);
        }
        token_choices[t] = choices;
        token_routers[t] = routers;
    }
    __syncthreads();
    for (int i = threadIdx.x; i <= K; i += blockDim.x)
        if (hist[i]) atomicAdd(&router_hist[i], (unsigned long long)hist[i]);
}

// one wave per sequence: exact integer sum of the tokens' differing routers, one division
__global__ void __launch_bounds__(256)
sequence_mean_kernel(int nseq, const int32_t *__restrict__ seq_offsets, const int32_t *__restrict__ token_routers,
                     double *__restrict__ seq_mean) {
    const int s = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (s >= nseq) return;
    const int lo = seq_offsets[s], hi = seq_offsets[s + 1];
    long long sum = 0;
    for (int t = lo + lane_id(); t < hi; t += kWave) sum += token_routers[t];
    sum = wave_sum(sum);
    if (lane_id() == 0) seq_mean[s] = hi > lo ? (double)sum / (double)(hi - lo) : 0.0;
}

// e^d - 1 - d = d^2 (1/2! + d/3! + d^2/4! + ...): for |d| <= 0.5 the series through d^14/16! is
// exact to double rounding (next term < 3e-19 of the first) and free of the cancellation that
// e^d - 1 - d suffers for small d; beyond, expm1(d) - d.  Most tokens have |log r| << 0.5, and the
// library expm1 alone kept this reduction at 3 percent of the memory rate.
__device__ __forceinline__ double k3_term(double d) {
    if (fabs(d) > 0.5) return expm1(d) - d;
    constexpr double c[15] = {5.00000000000000000e-01, 1.66666666666666657e-01, 4.16666666666666644e-02, 8.33333333333333322e-03, 1.38888888888888894e-03, 1.98412698412698413e-04, 2.48015873015873016e-05, 2.75573192239858925e-06, 2.75573192239858883e-07, 2.50521083854417202e-08, 2.08767569878681002e-09, 1.60590438368216133e-10, 1.14707455977297245e-11, 7.64716373181981641e-13, 4.77947733238738525e-14};
    double p = c[14];
#pragma unroll
    for (int k = 13; k >= 0; --k) p = fma(p, d, c[k]);
    return d * d * p;
}

struct TauArgs {
    float log_tau[kMaxTau];   // float(log(double(tau))); +inf beyond ntau
};

struct PolicyPartial {
    double k3;
    unsigned long long over[kMaxTau];
};

// log r = logp_train - logp_infer.  k3 term e^d - 1 - d in double (for |d| ~ 1e-3 the term is
// d^2/2 and would lose most of its digits in float), see k3_term(); the threshold test
// |log r| > log tau is taken in float on the float difference.
__global__ void __launch_bounds__(256)
policy_partial_kernel(int64_t n, const float *__restrict__ lt, const float *__restrict__ li, TauArgs taus,
                      PolicyPartial *__restrict__ part) {
    float thr[kMaxTau];
#pragma unroll
    for (int i = 0; i < kMaxTau; ++i) thr[i] = taus.log_tau[i];
    double k3 = 0.0;
    int over[kMaxTau];
#pragma unroll
    for (int i = 0; i < kMaxTau; ++i) over[i] = 0;
    auto one = [&](float a, float b) {
        const double d = (double)a - (double)b;
        k3 += k3_term(d);
        const float ad = fabsf(a - b);
#pragma unroll
        for (int j = 0; j < kMaxTau; ++j) over[j] += ad > thr[j];
    };
    // 16-byte loads when both arrays allow it (the order of a thread's terms is fixed either way)
    const bool vec = (((uintptr_t)lt | (uintptr_t)li) & 15) == 0;
    const int64_t n4 = vec ? n / 4 : 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
        const float4 a = ((const float4 *)lt)[i], b = ((const float4 *)li)[i];
        one(a.x, b.x);
        one(a.y, b.y);
        one(a.z, b.z);
        one(a.w, b.w);
    }
    for (int64_t i = 4 * n4 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        one(lt[i], li[i]);
    __shared__ double sk[4];
    __shared__ int so[4][kMaxTau];
    const int w = threadIdx.x / kWave;
    k3 = wave_sum(k3);
#pragma unroll
    for (int j = 0; j < kMaxTau; ++j) over[j] = wave_sum(over[j]);
    if (lane_id() == 0) {
        sk[w] = k3;
#pragma unroll
        for (int j = 0; j < kMaxTau; ++j) so[w][j] = over[j];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        PolicyPartial p;
        p.k3 = (sk[0] + sk[1]) + (sk[2] + sk[3]);
        for (int j = 0; j < kMaxTau; ++j) p.over[j] = (unsigned long long)(so[0][j] + so[1][j] + so[2][j] + so[3][j]);
        part[blockIdx.x] = p;
    }
}

// fixed-order sum of the block partials: 64 threads take contiguous runs, thread 0 adds the 64 runs
__global__ void __launch_bounds__(64)
policy_final_kernel(int64_t n, int nblocks, int ntau, const PolicyPartial *__restrict__ part, double *__restrict__ kl,
                    double *__restrict__ frac) {
    __shared__ double sk[64];
    __shared__ unsigned long long so[64][kMaxTau];
    const int per = (nblocks + 63) / 64;
    const int b0 = threadIdx.x * per, b1 = min(nblocks, b0 + per);
    double s = 0.0;
    unsigned long long c[kMaxTau];
    for (int j = 0; j < kMaxTau; ++j) c[j] = 0;
    for (int b = b0; b < b1; ++b) {
        s += part[b].k3;
        for (int j = 0; j < kMaxTau; ++j) c[j] += part[b].over[j];
    }
    sk[threadIdx.x] = s;
    for (int j = 0; j < kMaxTau; ++j) so[threadIdx.x][j] = c[j];
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < 64; ++i) t += sk[i];
        *kl = n > 0 ? t / (double)n : 0.0;
    }
    if ((int)threadIdx.x < ntau) {
        unsigned long long t = 0;
        for (int i = 0; i < 64; ++i) t += so[i][threadIdx.x];
        frac[threadIdx.x] = n > 0 ? (double)t / (double)n : 0.0;
    }
}

}  // namespace

size_t policy_ws_bytes() { return align_up((size_t)kDiagBlocks * sizeof(PolicyPartial), 256); }
int policy_max_tau() { return kMaxTau; }

hipError_t launch_routing_diff(int T, int K, int L, const void *a, const void *b, int idx_dtype, int64_t token_stride,
                               int64_t layer_stride, const int32_t *seq_offsets, int nseq, int64_t *router_hist,
                               int32_t *token_choices, int32_t *token_routers, double *seq_mean, hipStream_t s) {
    {
        ProfScope ps(PROF_ROUTING_DIFF, s);
        const int grid = (T + 255) / 256;
        if (idx_dtype == R3_IDX_U8)
            routing_diff_kernel<uint8_t><<<grid, 256, 0, s>>>(T, K, L, (const uint8_t *)a, (const uint8_t *)b,
                                                             token_stride, layer_stride,
                                                             (unsigned long long *)router_hist, token_choices,
                                                             token_routers);
        else
            routing_diff_kernel<uint16_t><<<grid, 256, 0, s>>>(T, K, L, (const uint16_t *)a, (const uint16_t *)b,
                                                              token_stride, layer_stride,
                                                              (unsigned long long *)router_hist, token_choices,
                                                              token_routers);
    }
    if (seq_mean && nseq > 0)
        sequence_mean_kernel<<<(nseq + 3) / 4, 256, 0, s>>>(nseq, seq_offsets, token_routers, seq_mean);
    return hipGetLastError();
}

hipError_t launch_policy_discrepancy(int64_t n, const float *lt, const float *li, int ntau, const float *tau_host,
                                     double *kl, double *frac, void *ws, hipStream_t s) {
    PolicyPartial *part = (PolicyPartial *)ws;
    TauArgs taus;
    for (int i = 0; i < kMaxTau; ++i) taus.log_tau[i] = i < ntau ? (float)log((double)tau_host[i]) : INFINITY;
    int64_t want = (n + 1023) / 1024;
    const int blocks = (int)(want < 1 ? 1 : (want > kDiagBlocks ? kDiagBlocks : want));
    ProfScope ps(PROF_POLICY, s);
    policy_partial_kernel<<<blocks, 256, 0, s>>>(n, lt, li, taus, part);
    policy_final_kernel<<<1, 64, 0, s>>>(n, blocks, ntau, part, kl, frac);
    return hipGetLastError();
}

}  // namespace r3
