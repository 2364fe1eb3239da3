// Routing kernels of the replayed MoE layer (arxiv 2510.11370, Section 4.1):
// TopKMask record, replay gate, dispatch permutation, weighted combine, and the
// element-wise parts of the backward.  All of them are bound by HBM traffic, so
// they move 16-byte vectors per lane, read every input once and use wave-level
// reductions; none uses floating-point atomics (results are bit-reproducible).
#include "r3_kernels.h"
#include "r3_topk.h"

namespace r3 {

// ---------------------------------------------------------------------------
// TopKMask
// ---------------------------------------------------------------------------
// Fast record: 8 lanes per token (8 tokens per wave), K <= 8, E <= 512.
// Lane `sub` of a token owns the contiguous id range [sub*EPL, (sub+1)*EPL) and keeps its 8
// largest keys in a sorted register list; three butterfly rounds of bitonic merges leave every
// lane with the token's 8 largest keys.  The K-th of them is the threshold: keys above it are
// taken, keys equal to it are taken lowest id first until K are out (prefix counts over the
// 8 lanes give each lane its quota and its output position, so ids come out ascending).
template <typename IdxT>
__global__ void __launch_bounds__(256)
record_topk_sub8_kernel(int T, int E, int K, int EPL, const float *__restrict__ logits, int64_t ld,
                        IdxT *__restrict__ idx, int64_t stride, int32_t *status) {
    const int t = blockIdx.x * 32 + (int)(threadIdx.x >> 3);
    const int sub = threadIdx.x & 7;
    const bool live = t < T;
    const float *row = logits + (int64_t)(live ? t : 0) * ld;
    const int e0 = sub * EPL;
    uint32_t top[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) top[j] = 0u;
    bool bad = false;
    for (int i = 0; i < EPL; ++i) {
        const int e = e0 + i;
        uint32_t v = 0u;
        if (live && e < E) {
            bool nf;
            v = order_key(row[e], nf);
            bad |= nf;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t hi = max(top[j], v);
            v = min(top[j], v);
            top[j] = hi;
        }
    }
    // butterfly merge over the token's 8 lanes: max(mine[i], partner[7-i]) is the top 8 of the
    // union as a bitonic sequence; three compare-exchange stages sort it again
#pragma unroll
    for (int m = 1; m < 8; m <<= 1) {
        uint32_t other[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) other[j] = __shfl_xor(top[j], m, 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) top[j] = max(top[j], other[7 - j]);
        cmpx_desc(top[0], top[4]); cmpx_desc(top[1], top[5]); cmpx_desc(top[2], top[6]); cmpx_desc(top[3], top[7]);
        cmpx_desc(top[0], top[2]); cmpx_desc(top[1], top[3]); cmpx_desc(top[4], top[6]); cmpx_desc(top[5], top[7]);
        cmpx_desc(top[0], top[1]); cmpx_desc(top[2], top[3]); cmpx_desc(top[4], top[5]); cmpx_desc(top[6], top[7]);
    }
    uint32_t thr = 0u;
    int above = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j == K - 1) thr = top[j];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j < K && top[j] > thr) ++above;
    // second pass over the lane's own ids
    int n_gt = 0, n_eq = 0;
    for (int i = 0; i < EPL; ++i) {
        const int e = e0 + i;
        if (live && e < E) {
            bool nf;
            const uint32_t v = order_key(row[e], nf);
            n_gt += v > thr;
            n_eq += v == thr;
        }
    }
    // exclusive prefix over the 8 lanes (ids ascend with the lane)
    int eq_before = n_eq, gt_before = n_gt;
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
        const int a = __shfl_up(eq_before, o, 8), b = __shfl_up(gt_before, o, 8);
        if (sub >= o) {
            eq_before += a;
            gt_before += b;
        }
    }
    eq_before -= n_eq;
    gt_before -= n_gt;
    const int quota = K - above;                                   // equal keys taken in all
    const int eq_taken_before = min(eq_before, quota);
    int my_quota = max(0, min(n_eq, quota - eq_before));           // equal keys this lane takes
    int pos = gt_before + eq_taken_before;
    if (live) {
        IdxT *out = idx + (int64_t)t * stride;
        for (int i = 0; i < EPL; ++i) {
            const int e = e0 + i;
            if (e < E) {
                bool nf;
                const uint32_t v = order_key(row[e], nf);
                bool take = v > thr;
                if (v == thr && my_quota > 0) {
                    take = true;
                    --my_quota;
                }
                if (take) out[pos++] = (IdxT)e;
            }
        }
        if (bad && status) atomicOr(status, R3_DATA_NONFINITE);
    }
}

// General record: one wave per token, rank counting, E <= 4096, K <= 64.
// key of element e beats key of element f if larger, or equal with lower id.
template <typename IdxT>
__global__ void __launch_bounds__(256)
record_topk_wave_kernel(int T, int E, int K, const float *__restrict__ logits, int64_t ld,
                        IdxT *__restrict__ idx, int64_t stride, int32_t *status) {
    extern __shared__ uint32_t keys_all[];
    const int w = threadIdx.x / kWave, lane = lane_id();
    const int t = blockIdx.x * 4 + w;
    uint32_t *keys = keys_all + w * E;
    bool bad = false;
    if (t < T)
        for (int e = lane; e < E; e += kWave) {
            bool nf;
            keys[e] = order_key(logits[(int64_t)t * ld + e], nf);
            bad |= nf;
        }
    __syncthreads();
    if (t >= T) return;
    int emitted = 0;  // wave-uniform
    for (int base = 0; base < E; base += kWave) {
        int e = base + lane;
        bool sel = false;
        if (e < E) {
            uint32_t mine = keys[e];
            int ahead = 0;
            for (int f = 0; f < E; ++f) {
                uint32_t kf = keys[f];
                ahead += (kf > mine || (kf == mine && f < e)) ? 1 : 0;
            }
            sel = ahead < K;
        }
        uint64_t m = __ballot(sel);
        if (sel) {
            int pos = emitted + __popcll(m & ((1ull << lane) - 1ull));
            idx[(int64_t)t * stride + pos] = (IdxT)e;
        }
        emitted += __popcll(m);
    }
    if (__ballot(bad) && lane == 0 && status) atomicOr(status, R3_DATA_NONFINITE);
}

// The same selection for E = 32 NV with vector loads and one pass over the row: the 8 lanes of a
// token read consecutive float4 pieces (lane `sub` holds ids 32 i + 4 sub + c, i < NV, c < 4: one
// 128-byte segment per token per load instruction), keep the keys in registers, and after the
// merges express "above the threshold" and "equal to it" as E-bit masks, OR-ed over the 8 lanes.
// The recorded set is the first mask plus the lowest-id bits of the second up to K; lane `sub`
// writes its sub-th set bit, so the K ids land ascending in one 8-byte segment.
template <typename IdxT, int NV>
__global__ void __launch_bounds__(256)
record_topk_vec_kernel(int T, int K, const float *__restrict__ logits, int64_t ld, IdxT *__restrict__ idx,
                       int64_t stride, int32_t *status) {
    const int t = blockIdx.x * 32 + (int)(threadIdx.x >> 3);
    const int sub = threadIdx.x & 7;
    const bool live = t < T;
    const float4 *row = (const float4 *)(logits + (int64_t)(live ? t : 0) * ld);
    uint32_t key[NV][4];
    bool bad = false;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const float4 v = row[i * 8 + sub];
        bool nf;
        key[i][0] = order_key(v.x, nf); bad |= nf;
        key[i][1] = order_key(v.y, nf); bad |= nf;
        key[i][2] = order_key(v.z, nf); bad |= nf;
        key[i][3] = order_key(v.w, nf); bad |= nf;
    }
    uint32_t gt[NV];
    topk_mask8<NV>(key, K, sub, gt);
    // lane `sub` emits the sub-th selected id
    int want = sub, id = -1;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        uint32_t w = gt[i];
        const int c = __popc(w);
        if (id < 0) {
            if (want < c) {
                for (int j = 0; j < want; ++j) w &= w - 1u;
                id = 32 * i + __ffs((int)w) - 1;
            } else {
                want -= c;
            }
        }
    }
    if (live) {
        if (sub < K && id >= 0) idx[(int64_t)t * stride + sub] = (IdxT)id;
        if (bad && status) atomicOr(status, R3_DATA_NONFINITE);
    }
}

template <typename IdxT>
static bool launch_record_vec(int T, int E, int K, const float *logits, int64_t ld, IdxT *idx, int64_t stride,
                              int32_t *status, hipStream_t s) {
    if (K > 8 || E % 32 != 0 || ld % 4 != 0 || ((uintptr_t)logits & 15)) return false;
    const int grid = (T + 31) / 32;
    switch (E / 32) {
        case 2: record_topk_vec_kernel<IdxT, 2><<<grid, 256, 0, s>>>(T, K, logits, ld, idx, stride, status); return true;
        case 4: record_topk_vec_kernel<IdxT, 4><<<grid, 256, 0, s>>>(T, K, logits, ld, idx, stride, status); return true;
        case 8: record_topk_vec_kernel<IdxT, 8><<<grid, 256, 0, s>>>(T, K, logits, ld, idx, stride, status); return true;
        default: return false;
    }
}

hipError_t launch_record_topk(int T, int E, int K, const float *logits, int64_t ld, void *idx,
                              int idx_dtype, int64_t stride, int32_t *status, hipStream_t s) {
    ProfScope ps(PROF_RECORD, s);
    if (idx_dtype == R3_IDX_U8 ? launch_record_vec(T, E, K, logits, ld, (uint8_t *)idx, stride, status, s)
                               : launch_record_vec(T, E, K, logits, ld, (uint16_t *)idx, stride, status, s))
        return hipGetLastError();
    if (K <= 8 && E <= 512) {
        const int EPL = (E + 7) / 8;
        const int grid = (T + 31) / 32;
        if (idx_dtype == R3_IDX_U8)
            record_topk_sub8_kernel<uint8_t><<<grid, 256, 0, s>>>(T, E, K, EPL, logits, ld, (uint8_t *)idx, stride,
                                                                 status);
        else
            record_topk_sub8_kernel<uint16_t><<<grid, 256, 0, s>>>(T, E, K, EPL, logits, ld, (uint16_t *)idx,
                                                                  stride, status);
    } else {
        size_t lds = (size_t)4 * E * sizeof(uint32_t);
        int grid = (T + 3) / 4;
        if (idx_dtype == R3_IDX_U8)
            record_topk_wave_kernel<uint8_t><<<grid, 256, lds, s>>>(T, E, K, logits, ld, (uint8_t *)idx,
                                                                   stride, status);
        else
            record_topk_wave_kernel<uint16_t><<<grid, 256, lds, s>>>(T, E, K, logits, ld,
                                                                    (uint16_t *)idx, stride, status);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Replay gate from logits in memory: one thread per token.
// g_j = exp(s[idx_j] - m) / sum_i exp(s[idx_i] - m), m = max over the set.
// ---------------------------------------------------------------------------
template <typename IdxT>
__global__ void __launch_bounds__(256)
gate_kernel(int T, int E, int K, const float *__restrict__ logits, const IdxT *__restrict__ idx,
            int64_t stride, float *__restrict__ gates, int32_t *status) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const IdxT *id = idx + (int64_t)t * stride;
    const float *row = logits + (int64_t)t * E;
    float m = -INFINITY;
    int bad = 0;
    for (int j = 0; j < K; ++j) {
        int e = (int)id[j];
        if (e >= E) {
            bad |= R3_DATA_IDX_RANGE;
            e = E - 1;
        }
        const float z = row[e];
        if (!(fabsf(z) <= 3.4028235e38f)) bad |= R3_DATA_NONFINITE;
        m = fmaxf(m, z);
    }
    float den = 0.0f;
    for (int j = 0; j < K; ++j) {
        int e = min((int)id[j], E - 1);
        float p = expf(row[e] - m);
        gates[(int64_t)t * K + j] = p;
        den += p;
    }
    float inv = 1.0f / den;
    for (int j = 0; j < K; ++j) gates[(int64_t)t * K + j] *= inv;
    if (bad && status) atomicOr(status, bad);
}

hipError_t launch_gate(int T, int E, int K, const float *logits, const void *idx, int idx_dtype,
                       int64_t stride, float *gates, int32_t *status, hipStream_t s) {
    ProfScope ps(PROF_GATE, s);
    int grid = (T + 255) / 256;
    if (idx_dtype == R3_IDX_U8)
        gate_kernel<uint8_t><<<grid, 256, 0, s>>>(T, E, K, logits, (const uint8_t *)idx, stride, gates, status);
    else
        gate_kernel<uint16_t><<<grid, 256, 0, s>>>(T, E, K, logits, (const uint16_t *)idx, stride, gates, status);
    return hipGetLastError();
}

// Routing agreement (Section 3.2, router level): per token compare the top-K
// set of the training logits with the recorded set.  A wave takes a token at a
// time: its E order keys sit in the wave's LDS strip, and for each recorded
// expert all 64 lanes count the keys ahead of it (one ballot per 64 experts).
// A wave walks many tokens and a block adds its totals once: agree[0] += tokens
// with equal sets, agree[1] += shared experts.  Integer atomics only.
template <typename IdxT>
__global__ void __launch_bounds__(256)
agreement_kernel(int T, int E, int K, const float *__restrict__ logits, const IdxT *__restrict__ idx,
                 int64_t stride, unsigned long long *agree) {
    extern __shared__ uint32_t keys_all[];
    __shared__ unsigned long long part[4][2];
    const int w = threadIdx.x / kWave, lane = lane_id();
    uint32_t *keys = keys_all + w * E;
    unsigned long long equal = 0, common = 0;
    for (int t = blockIdx.x * 4 + w; t < T; t += gridDim.x * 4) {
        for (int e = lane; e < E; e += kWave) {
            bool nf;
            keys[e] = order_key(logits[(int64_t)t * E + e], nf);
        }
        // one wave's LDS writes are complete before its later LDS reads
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_wave_barrier();
        int shared = 0;
        for (int j = 0; j < K; ++j) {
            const int e = min((int)idx[(int64_t)t * stride + j], E - 1);
            const uint32_t mine = keys[e];
            int ahead = 0;
            for (int f0 = 0; f0 < E; f0 += kWave) {
                const int f = f0 + lane;
                const uint32_t kf = f < E ? keys[f] : 0u;
                const bool before = f < E && (kf > mine || (kf == mine && f < e));
                ahead += __popcll(__ballot(before));
            }
            shared += ahead < K;
        }
        common += (unsigned long long)shared;
        equal += shared == K;
        __builtin_amdgcn_wave_barrier();   // the strip is rewritten for the next token
    }
    if (lane == 0) {
        part[w][0] = equal;
        part[w][1] = common;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long a0 = 0, a1 = 0;
        for (int i = 0; i < 4; ++i) {
            a0 += part[i][0];
            a1 += part[i][1];
        }
        if (a1) atomicAdd(agree + 1, a1);
        if (a0) atomicAdd(agree, a0);
    }
}

hipError_t launch_agreement(int T, int E, int K, const float *logits, const void *idx, int idx_dtype,
                            int64_t stride, int64_t *agree, hipStream_t s) {
    ProfScope ps(PROF_AGREEMENT, s);
    size_t lds = (size_t)4 * E * sizeof(uint32_t);
    int grid = (T + 3) / 4;
    if (grid > 2048) grid = 2048;
    if (idx_dtype == R3_IDX_U8)
        agreement_kernel<uint8_t><<<grid, 256, lds, s>>>(T, E, K, logits, (const uint8_t *)idx, stride,
                                                        (unsigned long long *)agree);
    else
        agreement_kernel<uint16_t><<<grid, 256, lds, s>>>(T, E, K, logits, (const uint16_t *)idx, stride,
                                                         (unsigned long long *)agree);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Dispatch permutation: stable counting sort of the T*K slots by expert.
//   pass 1: per-chunk expert histograms (one wave per chunk of slots)
//   pass 2: exclusive scan over (expert, chunk) -> offsets and chunk bases
//   pass 3: every wave walks its chunk in slot order and places slots
//   pass 4: row gather, one read of x[t] feeding its K destination rows
// The placement never depends on arrival order, so perm is unique.
// ---------------------------------------------------------------------------
// A wave's chunk is walked 64 slots at a time, kPermBatch such steps per batch: the ids of a whole
// batch are fetched before any of them is used, so the wave pays one memory round trip per batch
// instead of one per step.
constexpr int kPermBatch = 16;
// slot -> (token, position) in 32-bit arithmetic (T*K < 2^31), a shift when K is a power of two:
// a 64-bit division by a run-time K is some hundred instructions, and these kernels did two per slot
struct SlotSplit {
    int K, shift;
    __device__ __forceinline__ explicit SlotSplit(int K_) : K(K_), shift((K_ & (K_ - 1)) == 0 ? __ffs(K_) - 1 : -1) {}
    __device__ __forceinline__ void operator()(int sl, int &t, int &j) const {
        if (shift >= 0) {
            t = sl >> shift;
            j = sl & (K - 1);
        } else {
            t = (int)((unsigned)sl / (unsigned)K);
            j = sl - t * K;
        }
    }
};
constexpr int kWaitLds = 15 | (7 << 4) | (0 << 8) | (3 << 14);   // s_waitcnt lgkmcnt(0): LDS only, not the stores

template <typename IdxT>
__global__ void __launch_bounds__(256)
permute_hist_kernel(int T, int E, int K, const IdxT *__restrict__ idx, int64_t stride, int chunk,
                    int nchunks, int32_t *__restrict__ chunk_hist, int32_t *status) {
    extern __shared__ int32_t hist_all[];
    const int w = threadIdx.x / kWave, lane = lane_id();
    const int c = blockIdx.x * 4 + w;
    int32_t *hist = hist_all + w * E;
    for (int e = lane; e < E; e += kWave) hist[e] = 0;
    __syncthreads();
    if (c >= nchunks) return;
    const int S = T * K, s0 = c * chunk;
    const SlotSplit split(K);
    // a token's K ids sit in K neighbouring lanes of one step when K divides 64 (chunks start at
    // multiples of 64): then the duplicate check compares lanes instead of loading ids again
    const bool lanes_hold_token = 64 % K == 0;
    int bad = 0;
    for (int i0 = 0; i0 < chunk; i0 += kWave * kPermBatch) {
        int ev[kPermBatch];
#pragma unroll
        for (int u = 0; u < kPermBatch; ++u) {
            const int sl = s0 + i0 + u * kWave + lane;
            ev[u] = -1;
            if (i0 + u * kWave < chunk && sl < S) {
                int t, j;
                split(sl, t, j);
                ev[u] = (int)idx[(int64_t)t * stride + j];
            }
        }
#pragma unroll
        for (int u = 0; u < kPermBatch; ++u) {
            const int sl = s0 + i0 + u * kWave + lane;
            int e = ev[u];
            const bool live = e >= 0;
            if (live && e >= E) {
                bad |= R3_DATA_IDX_RANGE;
                e = E - 1;
            }
            if (lanes_hold_token) {
                const int j = lane % K;   // (sl % K: chunk starts and steps are multiples of 64)
                for (int back = 1; back < K; ++back) {
                    const int other = __shfl(e, lane - back);
                    if (live && back <= j && other == e) bad |= R3_DATA_IDX_DUP;
                }
            } else if (live) {
                int t, j;
                split(sl, t, j);
                for (int jj = 0; jj < j; ++jj)
                    if (min((int)idx[(int64_t)t * stride + jj], E - 1) == e) bad |= R3_DATA_IDX_DUP;
            }
            if (live) atomicAdd(&hist[e], 1);
        }
    }
    // LDS atomics of one wave are complete before its later LDS reads
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();
    for (int e = lane; e < E; e += kWave) chunk_hist[(int64_t)c * E + e] = hist[e];
    if (bad && status) atomicOr(status, bad);
}

// One block of 1024 threads.  chunk_base [nchunks,E] receives the exclusive running count of
// chunk_hist over chunks; counts/offsets are written.  An expert's column of chunk_hist is shared out
// among G = 1024 / E' threads (E' = E rounded up to a power of two), each taking a contiguous range of
// chunks: sums of the ranges first, then every thread walks its range again from its own base.  (One
// thread per expert walking all chunks paid a memory round trip per 8 chunks, 16 in a row at 128
// chunks, with 7 of 8 threads idle at E = 128.)
__global__ void __launch_bounds__(1024)
permute_scan_kernel(int E, int nchunks, const int32_t *__restrict__ chunk_hist, int32_t *__restrict__ chunk_base,
                    int32_t *__restrict__ counts, int32_t *__restrict__ offsets) {
    __shared__ int32_t tot[kMaxE];
    __shared__ int32_t part[1024];
    int Ep = 1;
    while (Ep < E && Ep < 1024) Ep <<= 1;
    const int G = E <= 1024 ? 1024 / Ep : 1;                 // threads per expert
    const int per_g = (nchunks + G - 1) / G;                 // chunks per thread
    const int g = E <= 1024 ? threadIdx.x / Ep : 0;
    const int c0 = min(g * per_g, nchunks), c1 = min(c0 + per_g, nchunks);
    auto walk = [&](int e, int32_t run, bool write) {
        int c = c0;
        for (; c + 8 <= c1; c += 8) {
            int32_t h[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) h[u] = chunk_hist[(int64_t)(c + u) * E + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (write) chunk_base[(int64_t)(c + u) * E + e] = run;
                run += h[u];
            }
        }
        for (; c < c1; ++c) {
            const int32_t h = chunk_hist[(int64_t)c * E + e];
            if (write) chunk_base[(int64_t)c * E + e] = run;
            run += h;
        }
        return run;
    };
    if (E <= 1024) {
        const int e = threadIdx.x % Ep;
        part[threadIdx.x] = e < E ? walk(e, 0, false) : 0;
        __syncthreads();
        int32_t base = 0, all = 0;
        for (int gg = 0; gg < G; ++gg) {
            const int32_t v = part[gg * Ep + e];
            base += gg < g ? v : 0;
            all += v;
        }
        if (e < E) {
            walk(e, base, true);
            if (g == 0) {
                tot[e] = all;
                counts[e] = all;
            }
        }
    } else {
        for (int e = threadIdx.x; e < E; e += blockDim.x) {
            const int32_t all = walk(e, 0, true);
            tot[e] = all;
            counts[e] = all;
        }
    }
    __syncthreads();
    // exclusive scan of tot[0..E): each thread owns a contiguous span
    const int per = (E + blockDim.x - 1) / blockDim.x;
    const int b = threadIdx.x * per;
    int32_t sum = 0;
    for (int i = 0; i < per; ++i)
        if (b + i < E) sum += tot[b + i];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int o = 1; o < (int)blockDim.x; o <<= 1) {
        int32_t v = (threadIdx.x >= (unsigned)o) ? part[threadIdx.x - o] : 0;
        __syncthreads();
        part[threadIdx.x] += v;
        __syncthreads();
    }
    int32_t run = part[threadIdx.x] - sum;
    for (int i = 0; i < per; ++i)
        if (b + i < E) {
            offsets[b + i] = run;
            run += tot[b + i];
        }
    if (threadIdx.x == blockDim.x - 1) offsets[E] = part[threadIdx.x];
}

template <typename IdxT>
__global__ void __launch_bounds__(256)
permute_place_kernel(int T, int E, int K, const IdxT *__restrict__ idx, int64_t stride, int chunk,
                     int nchunks, const int32_t *__restrict__ chunk_base,
                     const int32_t *__restrict__ offsets, int32_t *__restrict__ inv_perm,
                     int32_t *__restrict__ perm) {
    extern __shared__ int32_t cnt_all[];
    const int w = threadIdx.x / kWave, lane = lane_id();
    const int c = blockIdx.x * 4 + w;
    int32_t *cnt = cnt_all + w * E;
    if (c < nchunks)
        for (int e = lane; e < E; e += kWave) cnt[e] = offsets[e] + chunk_base[(int64_t)c * E + e];
    __syncthreads();
    if (c >= nchunks) return;
    const int S = T * K, s0 = c * chunk;
    const SlotSplit split(K);
    int ebits = 1;
    while ((1 << ebits) < E) ++ebits;
    const uint64_t lt = (1ull << lane) - 1ull;
    for (int i0 = 0; i0 < chunk; i0 += kWave * kPermBatch) {
        int ev[kPermBatch];
#pragma unroll
        for (int u = 0; u < kPermBatch; ++u) {
            const int sl = s0 + i0 + u * kWave + lane;
            ev[u] = -1;
            if (i0 + u * kWave < chunk && sl < S) {
                int t, j;
                split(sl, t, j);
                ev[u] = min((int)idx[(int64_t)t * stride + j], E - 1);
            }
        }
#pragma unroll
        for (int u = 0; u < kPermBatch; ++u) {
            const int sl = s0 + i0 + u * kWave + lane;
            const bool live = ev[u] >= 0;
            const int e = live ? ev[u] : 0;
            // lanes holding the same expert
            uint64_t same = __ballot(live);
            for (int b = 0; b < ebits; ++b) {
                uint64_t bal = __ballot((e >> b) & 1);
                same &= ((e >> b) & 1) ? bal : ~bal;
            }
            if (live) {
                int row = cnt[e] + __popcll(same & lt);
                inv_perm[sl] = row;
                perm[row] = (int32_t)sl;
            }
            // (LDS traffic only: the stores above need not have landed)
            __builtin_amdgcn_s_waitcnt(kWaitLds);
            __builtin_amdgcn_wave_barrier();
            // the highest lane of each group advances the group's counter
            if (live && (same >> lane) == 1ull) cnt[e] += __popcll(same);
            __builtin_amdgcn_s_waitcnt(kWaitLds);
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// 16-byte load of data that is read once per launch: marked non-temporal, so that the rows are not
// kept in L2 (measured: the gathered-row reads of combine run 20 % faster; the same hint on stores
// was slower)
template <typename V> __device__ __forceinline__ V ld_once(const V *p) {
    if constexpr (sizeof(V) == 16) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        return __builtin_bit_cast(V, __builtin_nontemporal_load((const u32x4 *)p));
    } else {
        return *p;
    }
}

// Row gather by token: the block reads x[t] once and writes its K copies.
// V is the vector type moved per thread (uint4 when rows are 16-byte multiples).
template <typename V>
__global__ void __launch_bounds__(256)
gather_rows_kernel(int T, int K, int row_vecs, const V *__restrict__ x,
                   const int32_t *__restrict__ inv_perm, V *__restrict__ Xp) {
    const int t = blockIdx.x;
    __shared__ int32_t rows[kMaxK];
    if (threadIdx.x < (unsigned)K) rows[threadIdx.x] = inv_perm[(int64_t)t * K + threadIdx.x];
    __syncthreads();
    for (int c = threadIdx.x; c < row_vecs; c += blockDim.x) {
        V v = x[(int64_t)t * row_vecs + c];
        for (int j = 0; j < K; ++j) Xp[(int64_t)rows[j] * row_vecs + c] = v;
    }
}

static int pick_chunk(int64_t S) {
    // slots per wave-chunk: at least 1024, at most 512 chunks in total
    int64_t c = 1024;
    while ((S + c - 1) / c > 512) c *= 2;
    return (int)c;
}

size_t permute_ws_bytes(int T, int E, int K) {
    int64_t S = (int64_t)T * K;
    int chunk = pick_chunk(S);
    int64_t nchunks = (S + chunk - 1) / chunk;
    return 2 * align_up((size_t)nchunks * E * sizeof(int32_t), 256);  // histograms + running bases
}

hipError_t launch_permute(int T, int d, int E, int K, int elem_bytes, const void *x, const void *idx,
                          int idx_dtype, int64_t stride, int32_t *counts, int32_t *offsets,
                          int32_t *inv_perm, int32_t *perm, void *Xp, int32_t *status, void *ws,
                          hipStream_t s) {
    const int64_t S = (int64_t)T * K;
    const int chunk = pick_chunk(S);
    const int nchunks = (int)((S + chunk - 1) / chunk);
    int32_t *chunk_hist = (int32_t *)ws;
    int32_t *chunk_base = (int32_t *)((char *)ws + align_up((size_t)nchunks * E * sizeof(int32_t), 256));
    const int grid = (nchunks + 3) / 4;
    const size_t lds = (size_t)4 * E * sizeof(int32_t);
    {
    ProfScope ps(PROF_PERMUTE_INDEX, s);
    if (idx_dtype == R3_IDX_U8)
        permute_hist_kernel<uint8_t><<<grid, 256, lds, s>>>(T, E, K, (const uint8_t *)idx, stride, chunk,
                                                           nchunks, chunk_hist, status);
    else
        permute_hist_kernel<uint16_t><<<grid, 256, lds, s>>>(T, E, K, (const uint16_t *)idx, stride,
                                                            chunk, nchunks, chunk_hist, status);
    permute_scan_kernel<<<1, 1024, 0, s>>>(E, nchunks, chunk_hist, chunk_base, counts, offsets);
    if (idx_dtype == R3_IDX_U8)
        permute_place_kernel<uint8_t><<<grid, 256, lds, s>>>(T, E, K, (const uint8_t *)idx, stride, chunk,
                                                            nchunks, chunk_base, offsets, inv_perm, perm);
    else
        permute_place_kernel<uint16_t><<<grid, 256, lds, s>>>(T, E, K, (const uint16_t *)idx, stride,
                                                             chunk, nchunks, chunk_base, offsets,
                                                             inv_perm, perm);
    }
    if (Xp) {
        ProfScope ps(PROF_GATHER_ROWS, s);
        const int64_t row_bytes = (int64_t)d * elem_bytes;
        if (row_bytes % 16 == 0)
            gather_rows_kernel<uint4><<<T, 256, 0, s>>>(T, K, (int)(row_bytes / 16), (const uint4 *)x,
                                                       inv_perm, (uint4 *)Xp);
        else if (row_bytes % 4 == 0)
            gather_rows_kernel<uint32_t><<<T, 256, 0, s>>>(T, K, (int)(row_bytes / 4),
                                                          (const uint32_t *)x, inv_perm, (uint32_t *)Xp);
        else
            gather_rows_kernel<uint16_t><<<T, 256, 0, s>>>(T, K, (int)(row_bytes / 2),
                                                          (const uint16_t *)x, inv_perm, (uint16_t *)Xp);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Combine: y[t] = sum_j g[t,j] * Yp[inv_perm[t*K+j]], j ascending, f32.
// One block per token; each thread owns VEC consecutive columns.
// ---------------------------------------------------------------------------
template <typename T, int VEC> struct VecIO;
template <> struct VecIO<bf16_t, 8> {
    typedef uint4 V;
    static __device__ __forceinline__ void unpack(const V &v, float *f) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ V pack(const float *f) {
        V v;
        v.x = pack_bf16x2(f[0], f[1]);
        v.y = pack_bf16x2(f[2], f[3]);
        v.z = pack_bf16x2(f[4], f[5]);
        v.w = pack_bf16x2(f[6], f[7]);
        return v;
    }
};
template <> struct VecIO<float, 4> {
    typedef float4 V;
    static __device__ __forceinline__ void unpack(const V &v, float *f) {
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    static __device__ __forceinline__ V pack(const float *f) { return make_float4(f[0], f[1], f[2], f[3]); }
};
template <> struct VecIO<bf16_t, 1> {
    typedef bf16_t V;
    static __device__ __forceinline__ void unpack(const V &v, float *f) { f[0] = bf16_to_f32(v); }
    static __device__ __forceinline__ V pack(const float *f) { return f32_to_bf16(f[0]); }
};
template <> struct VecIO<float, 1> {
    typedef float V;
    static __device__ __forceinline__ void unpack(const V &v, float *f) { f[0] = v; }
    static __device__ __forceinline__ V pack(const float *f) { return f[0]; }
};

// KT > 0: K known at compile time, so that a thread's K row loads are all in flight together
template <typename T, int VEC, int KT>
__global__ void __launch_bounds__(256)
combine_kernel(int Krt, int row_vecs, const typename VecIO<T, VEC>::V *__restrict__ Yp,
               const float *__restrict__ gates, const int32_t *__restrict__ inv_perm,
               typename VecIO<T, VEC>::V *__restrict__ y) {
    typedef VecIO<T, VEC> IO;
    const int K = KT > 0 ? KT : Krt;
    const int t = blockIdx.x;
    __shared__ int32_t rows[kMaxK];
    __shared__ float g[kMaxK];
    if (threadIdx.x < (unsigned)K) {
        rows[threadIdx.x] = inv_perm[(int64_t)t * K + threadIdx.x];
        g[threadIdx.x] = gates ? gates[(int64_t)t * K + threadIdx.x] : 1.0f;   // no gates: rows arrive gated
    }
    __syncthreads();
    for (int c = threadIdx.x; c < row_vecs; c += blockDim.x) {
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
        if constexpr (KT > 0) {
            typename IO::V v[KT];
#pragma unroll
            for (int j = 0; j < KT; ++j) v[j] = ld_once(&Yp[(int64_t)rows[j] * row_vecs + c]);
#pragma unroll
            for (int j = 0; j < KT; ++j) {   // fixed j order: the sum is the same for every launch shape
                float f[VEC];
                IO::unpack(v[j], f);
                const float gj = g[j];
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = fmaf(gj, f[i], acc[i]);
            }
        } else {
            for (int j = 0; j < K; ++j) {
                float f[VEC];
                IO::unpack(Yp[(int64_t)rows[j] * row_vecs + c], f);
                const float gj = g[j];
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = fmaf(gj, f[i], acc[i]);
            }
        }
        y[(int64_t)t * row_vecs + c] = IO::pack(acc);
    }
}

hipError_t launch_combine(int T, int d, int K, int act, const void *Yp, const float *gates,
                          const int32_t *inv_perm, void *y, hipStream_t s) {
    ProfScope ps(PROF_COMBINE, s);
    if (act == R3_BF16) {
        if (d % 8 == 0 && K == 8)
            combine_kernel<bf16_t, 8, 8><<<T, 256, 0, s>>>(K, d / 8, (const uint4 *)Yp, gates, inv_perm,
                                                          (uint4 *)y);
        else if (d % 8 == 0)
            combine_kernel<bf16_t, 8, 0><<<T, 256, 0, s>>>(K, d / 8, (const uint4 *)Yp, gates, inv_perm,
                                                          (uint4 *)y);
        else
            combine_kernel<bf16_t, 1, 0><<<T, 256, 0, s>>>(K, d, (const bf16_t *)Yp, gates, inv_perm,
                                                          (bf16_t *)y);
    } else {
        if (d % 4 == 0)
            combine_kernel<float, 4, 0><<<T, 256, 0, s>>>(K, d / 4, (const float4 *)Yp, gates, inv_perm,
                                                         (float4 *)y);
        else
            combine_kernel<float, 1, 0><<<T, 256, 0, s>>>(K, d, (const float *)Yp, gates, inv_perm,
                                                         (float *)y);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Backward through combine and masked softmax, one block per token:
//   dg_j = <dy_t, Yp[row_j]>,  dYp[row_j] = g_j * dy_t,
//   dz_j = g_j (dg_j - sum_i g_i dg_i).
// Writes dz [T,K] f32 and, when ds_dense != NULL, the dense row ds[t,:] (zero off
// the recorded set) that the router weight gradient contracts: [T,E] f32, or for
// bf16 activations [T,2E] holding dz as hi and lo bf16 halves.
// ---------------------------------------------------------------------------
template <typename T, int VEC, typename IdxT, int KT>
__global__ void __launch_bounds__(256)
gate_backward_kernel(int E, int Krt, int row_vecs, const typename VecIO<T, VEC>::V *__restrict__ dy,
                     const typename VecIO<T, VEC>::V *__restrict__ Yp, const float *__restrict__ gates,
                     const int32_t *__restrict__ inv_perm, const IdxT *__restrict__ idx, int64_t stride,
                     typename VecIO<T, VEC>::V *__restrict__ dYp, float *__restrict__ dz,
                     T *__restrict__ ds_dense, int gated) {
    typedef VecIO<T, VEC> IO;
    const int K = KT > 0 ? KT : Krt;
    const int t = blockIdx.x;
    const int nw = blockDim.x / kWave, w = threadIdx.x / kWave, lane = lane_id();
    __shared__ int32_t rows[kMaxK];
    __shared__ float g[kMaxK];
    __shared__ float part[4][kMaxK];
    __shared__ float dgs[kMaxK];
    if (threadIdx.x < (unsigned)K) {
        rows[threadIdx.x] = inv_perm[(int64_t)t * K + threadIdx.x];
        g[threadIdx.x] = gates[(int64_t)t * K + threadIdx.x];
    }
    // bf16 activations: ds is stored as a (hi, lo) pair of bf16 rows [hi(E) | lo(E)] so that the
    // router weight gradient sees dz to about 16 bits instead of 8
    const int dsw = (sizeof(T) == 2) ? 2 * E : E;
    if (ds_dense)
        for (int e = threadIdx.x; e < dsw; e += blockDim.x) Elem<T>::st(ds_dense + (int64_t)t * dsw + e, 0.0f);
    __syncthreads();
    if constexpr (KT > 0) {
        // dy is read once per column chunk and the K rows of Yp are all in flight together; per
        // thread and per j the products are summed in the same order as in the loop below
        float dot[KT];
#pragma unroll
        for (int j = 0; j < KT; ++j) dot[j] = 0.0f;
        for (int c = threadIdx.x; c < row_vecs; c += blockDim.x) {
            float a[VEC];
            IO::unpack(dy[(int64_t)t * row_vecs + c], a);
            typename IO::V v[KT];
#pragma unroll
            for (int j = 0; j < KT; ++j) v[j] = ld_once(&Yp[(int64_t)rows[j] * row_vecs + c]);
#pragma unroll
            for (int j = 0; j < KT; ++j) {
                float b[VEC], o[VEC];
                IO::unpack(v[j], b);
                const float gj = g[j];
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    dot[j] = fmaf(a[i], b[i], dot[j]);
                    o[i] = gj * a[i];
                }
                dYp[(int64_t)rows[j] * row_vecs + c] = IO::pack(o);
            }
        }
#pragma unroll
        for (int j = 0; j < KT; ++j) {
            const float dsum = wave_sum(dot[j]);
            if (lane == 0) part[w][j] = dsum;
        }
    } else {
        for (int j = 0; j < K; ++j) {
            float dot = 0.0f;
            const float gj = g[j];
            for (int c = threadIdx.x; c < row_vecs; c += blockDim.x) {
                float a[VEC], b[VEC], o[VEC];
                IO::unpack(dy[(int64_t)t * row_vecs + c], a);
                IO::unpack(Yp[(int64_t)rows[j] * row_vecs + c], b);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    dot = fmaf(a[i], b[i], dot);
                    o[i] = gj * a[i];
                }
                dYp[(int64_t)rows[j] * row_vecs + c] = IO::pack(o);
            }
            dot = wave_sum(dot);
            if (lane == 0) part[w][j] = dot;
        }
    }
    __syncthreads();
    if (threadIdx.x < (unsigned)K) {
        float v = 0.0f;
        for (int i = 0; i < nw; ++i) v += part[i][threadIdx.x];
        dgs[threadIdx.x] = v;
    }
    __syncthreads();
    if (threadIdx.x < (unsigned)K) {
        // gated: the rows of Yp are g o, so the dot products are already g_j dg_j
        float mix = 0.0f;
        for (int j = 0; j < K; ++j) mix = gated ? mix + dgs[j] : fmaf(g[j], dgs[j], mix);
        float v = gated ? dgs[threadIdx.x] - g[threadIdx.x] * mix : g[threadIdx.x] * (dgs[threadIdx.x] - mix);
        dz[(int64_t)t * K + threadIdx.x] = v;
        if (ds_dense) {
            int e = min((int)idx[(int64_t)t * stride + threadIdx.x], E - 1);
            T *row = ds_dense + (int64_t)t * dsw;
            Elem<T>::st(row + e, v);
            if (sizeof(T) == 2) Elem<T>::st(row + E + e, v - Elem<T>::ld(row + e));
        }
    }
}

template <typename T, int VEC>
static hipError_t gate_backward_dispatch(int Tn, int E, int K, int row_vecs, const void *dy, const void *Yp,
                                         const float *gates, const int32_t *inv_perm, const void *idx,
                                         int idx_dtype, int64_t stride, void *dYp, float *dz,
                                         void *ds_dense, int gated, hipStream_t s) {
    typedef typename VecIO<T, VEC>::V V;
    if (idx_dtype == R3_IDX_U8 && K == 8 && VEC > 1)
        gate_backward_kernel<T, VEC, uint8_t, 8><<<Tn, 256, 0, s>>>(E, K, row_vecs, (const V *)dy, (const V *)Yp,
                                                                  gates, inv_perm, (const uint8_t *)idx,
                                                                  stride, (V *)dYp, dz, (T *)ds_dense, gated);
    else if (idx_dtype == R3_IDX_U8)
        gate_backward_kernel<T, VEC, uint8_t, 0><<<Tn, 256, 0, s>>>(E, K, row_vecs, (const V *)dy, (const V *)Yp,
                                                                  gates, inv_perm, (const uint8_t *)idx,
                                                                  stride, (V *)dYp, dz, (T *)ds_dense, gated);
    else
        gate_backward_kernel<T, VEC, uint16_t, 0><<<Tn, 256, 0, s>>>(E, K, row_vecs, (const V *)dy,
                                                                   (const V *)Yp, gates, inv_perm,
                                                                   (const uint16_t *)idx, stride, (V *)dYp,
                                                                   dz, (T *)ds_dense, gated);
    return hipGetLastError();
}

hipError_t launch_gate_backward(int T, int d, int E, int K, int act, const void *dy, const void *Yp,
                                const float *gates, const int32_t *inv_perm, const void *idx,
                                int idx_dtype, int64_t stride, void *dYp, float *dz, void *ds_dense,
                                int gated, hipStream_t s) {
    ProfScope ps(PROF_GATE_BWD, s);
    if (act == R3_BF16) {
        if (d % 8 == 0)
            return gate_backward_dispatch<bf16_t, 8>(T, E, K, d / 8, dy, Yp, gates, inv_perm, idx, idx_dtype,
                                                     stride, dYp, dz, ds_dense, gated, s);
        return gate_backward_dispatch<bf16_t, 1>(T, E, K, d, dy, Yp, gates, inv_perm, idx, idx_dtype, stride,
                                                 dYp, dz, ds_dense, gated, s);
    }
    if (d % 4 == 0)
        return gate_backward_dispatch<float, 4>(T, E, K, d / 4, dy, Yp, gates, inv_perm, idx, idx_dtype,
                                                stride, dYp, dz, ds_dense, gated, s);
    return gate_backward_dispatch<float, 1>(T, E, K, d, dy, Yp, gates, inv_perm, idx, idx_dtype, stride, dYp,
                                            dz, ds_dense, gated, s);
}

// ---------------------------------------------------------------------------
// Masked-softmax backward when the expert-gradient GEMM has already formed the dot products: its
// epilogue leaves, for every row r, `nparts` partial sums whose total is w = g <dy_t, o_r> = g dg.
//   w_j = sum_p wpart[row_j][p] (p ascending),   dz_j = g_j (dg_j - sum_i g_i dg_i) = w_j - g_j sum_i w_i
// One thread per slot, a token's K slots in neighbouring lanes; a block owns 256 / KP tokens (KP = K
// rounded up to a power of two) and writes their dense ds rows [hi(E) | lo(E)] (bf16): zeros first,
// then the K entries of each token.
// ---------------------------------------------------------------------------
template <typename IdxT>
__global__ void __launch_bounds__(256)
gate_backward_parts_kernel(int T, int E, int K, int KP, int nparts, const float *__restrict__ wpart,
                           const float *__restrict__ gates, const int32_t *__restrict__ inv_perm,
                           const IdxT *__restrict__ idx, int64_t stride, float *__restrict__ dz,
                           bf16_t *__restrict__ ds) {
    const int tpb = 256 / KP;                       // tokens per block
    const int t0 = blockIdx.x * tpb;
    const int nt = min(tpb, T - t0);
    // zero this block's ds rows: nt * 2E bf16, contiguous, a multiple of 4 bytes
    uint32_t *z = (uint32_t *)(ds + (int64_t)t0 * 2 * E);
    for (int i = threadIdx.x; i < nt * E; i += 256) z[i] = 0u;
    const int tl = threadIdx.x / KP, j = threadIdx.x % KP;
    const int t = t0 + tl;
    const bool live = tl < nt && j < K;
    float w = 0.0f, g = 0.0f;
    int e = 0;
    if (live) {
        const int row = inv_perm[(int64_t)t * K + j];
        const float *p = wpart + (int64_t)row * nparts;
        for (int i = 0; i < nparts; ++i) w += p[i];
        g = gates[(int64_t)t * K + j];
        e = min((int)idx[(int64_t)t * stride + j], E - 1);
    }
    // sum of w over the token's slots, in a fixed order: KP neighbouring lanes (KP <= 64 divides 64)
    float mix = w;
    for (int o = 1; o < KP; o <<= 1) mix += __shfl_xor(mix, o, 64);
    __syncthreads();                                // the zeros are in before the entries go on top
    if (live) {
        const float v = w - g * mix;
        dz[(int64_t)t * K + j] = v;
        bf16_t *row = ds + (int64_t)t * 2 * E;
        const bf16_t hi = f32_to_bf16(v);
        row[e] = hi;
        row[E + e] = f32_to_bf16(v - bf16_to_f32(hi));
    }
}

hipError_t launch_gate_backward_parts(int T, int E, int K, int nparts, const float *wpart, const float *gates,
                                      const int32_t *inv_perm, const void *idx, int idx_dtype, int64_t stride,
                                      float *dz, void *ds_dense, hipStream_t s) {
    ProfScope ps(PROF_GATE_BWD, s);
    int KP = 1;
    while (KP < K) KP <<= 1;                        // K <= kMaxK = 64
    const int tpb = 256 / KP;
    const int grid = (T + tpb - 1) / tpb;
    if (idx_dtype == R3_IDX_U8)
        gate_backward_parts_kernel<uint8_t><<<grid, 256, 0, s>>>(T, E, K, KP, nparts, wpart, gates, inv_perm,
                                                                (const uint8_t *)idx, stride, dz, (bf16_t *)ds_dense);
    else
        gate_backward_parts_kernel<uint16_t><<<grid, 256, 0, s>>>(T, E, K, KP, nparts, wpart, gates, inv_perm,
                                                                 (const uint16_t *)idx, stride, dz,
                                                                 (bf16_t *)ds_dense);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Final input gradient, one block per token:
//   dx[t] = sum_j dXp[row_j]  +  sum_j dz[t,j] * W_r[:, idx_j]
// WrT is W_r transposed ([E,d], act dtype) so that the router term reads rows.
// ---------------------------------------------------------------------------
template <typename T, int VEC, typename IdxT, int KT>
__global__ void __launch_bounds__(256)
dx_finish_kernel(int E, int Krt, int row_vecs, const typename VecIO<T, VEC>::V *__restrict__ dXp,
                 const typename VecIO<T, VEC>::V *__restrict__ WrT, const float *__restrict__ dz,
                 const int32_t *__restrict__ inv_perm, const IdxT *__restrict__ idx, int64_t stride,
                 typename VecIO<T, VEC>::V *__restrict__ dx) {
    typedef VecIO<T, VEC> IO;
    const int K = KT > 0 ? KT : Krt;
    const int t = blockIdx.x;
    __shared__ int32_t rows[kMaxK];
    __shared__ int32_t ids[kMaxK];
    __shared__ float z[kMaxK];
    if (threadIdx.x < (unsigned)K) {
        rows[threadIdx.x] = inv_perm[(int64_t)t * K + threadIdx.x];
        ids[threadIdx.x] = min((int)idx[(int64_t)t * stride + threadIdx.x], E - 1);
        z[threadIdx.x] = dz[(int64_t)t * K + threadIdx.x];
    }
    __syncthreads();
    for (int c = threadIdx.x; c < row_vecs; c += blockDim.x) {
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
        if constexpr (KT > 0) {   // all 2K row loads in flight together; same summation order as below
            typename IO::V v[KT], w[KT];
#pragma unroll
            for (int j = 0; j < KT; ++j) v[j] = ld_once(&dXp[(int64_t)rows[j] * row_vecs + c]);
#pragma unroll
            for (int j = 0; j < KT; ++j) w[j] = WrT[(int64_t)ids[j] * row_vecs + c];
#pragma unroll
            for (int j = 0; j < KT; ++j) {
                float f[VEC];
                IO::unpack(v[j], f);
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += f[i];
            }
#pragma unroll
            for (int j = 0; j < KT; ++j) {
                float f[VEC];
                IO::unpack(w[j], f);
                const float zj = z[j];
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = fmaf(zj, f[i], acc[i]);
            }
        } else {
            for (int j = 0; j < K; ++j) {
                float f[VEC];
                IO::unpack(dXp[(int64_t)rows[j] * row_vecs + c], f);
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += f[i];
            }
            for (int j = 0; j < K; ++j) {
                float f[VEC];
                IO::unpack(WrT[(int64_t)ids[j] * row_vecs + c], f);
                const float zj = z[j];
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = fmaf(zj, f[i], acc[i]);
            }
        }
        dx[(int64_t)t * row_vecs + c] = IO::pack(acc);
    }
}

template <typename T, int VEC>
static hipError_t dx_finish_dispatch(int Tn, int E, int K, int row_vecs, const void *dXp, const void *WrT,
                                     const float *dz, const int32_t *inv_perm, const void *idx,
                                     int idx_dtype, int64_t stride, void *dx, hipStream_t s) {
    typedef typename VecIO<T, VEC>::V V;
    if (idx_dtype == R3_IDX_U8 && K == 8 && VEC > 1)
        dx_finish_kernel<T, VEC, uint8_t, 8><<<Tn, 256, 0, s>>>(E, K, row_vecs, (const V *)dXp, (const V *)WrT, dz,
                                                              inv_perm, (const uint8_t *)idx, stride, (V *)dx);
    else if (idx_dtype == R3_IDX_U8)
        dx_finish_kernel<T, VEC, uint8_t, 0><<<Tn, 256, 0, s>>>(E, K, row_vecs, (const V *)dXp, (const V *)WrT, dz,
                                                              inv_perm, (const uint8_t *)idx, stride, (V *)dx);
    else
        dx_finish_kernel<T, VEC, uint16_t, 0><<<Tn, 256, 0, s>>>(E, K, row_vecs, (const V *)dXp, (const V *)WrT,
                                                               dz, inv_perm, (const uint16_t *)idx, stride,
                                                               (V *)dx);
    return hipGetLastError();
}

hipError_t launch_dx_finish(int T, int d, int E, int K, int act, const void *dXp, const void *WrT,
                            const float *dz, const int32_t *inv_perm, const void *idx, int idx_dtype,
                            int64_t stride, void *dx, hipStream_t s) {
    ProfScope ps(PROF_DX_FINISH, s);
    if (act == R3_BF16) {
        if (d % 8 == 0)
            return dx_finish_dispatch<bf16_t, 8>(T, E, K, d / 8, dXp, WrT, dz, inv_perm, idx, idx_dtype, stride,
                                                 dx, s);
        return dx_finish_dispatch<bf16_t, 1>(T, E, K, d, dXp, WrT, dz, inv_perm, idx, idx_dtype, stride, dx, s);
    }
    if (d % 4 == 0)
        return dx_finish_dispatch<float, 4>(T, E, K, d / 4, dXp, WrT, dz, inv_perm, idx, idx_dtype, stride, dx,
                                            s);
    return dx_finish_dispatch<float, 1>(T, E, K, d, dXp, WrT, dz, inv_perm, idx, idx_dtype, stride, dx, s);
}

// transpose a small [R,C] matrix (W_r) into [C,R]
template <typename T>
__global__ void transpose_kernel(int R, int C, const T *__restrict__ in, T *__restrict__ out) {
    __shared__ T tile[32][33];
    int c = blockIdx.x * 32 + threadIdx.x, r0 = blockIdx.y * 32;
    for (int i = threadIdx.y; i < 32; i += blockDim.y)
        if (r0 + i < R && c < C) tile[i][threadIdx.x] = in[(int64_t)(r0 + i) * C + c];
    __syncthreads();
    int r = r0 + threadIdx.x, c0 = blockIdx.x * 32;
    for (int i = threadIdx.y; i < 32; i += blockDim.y)
        if (c0 + i < C && r < R) out[(int64_t)(c0 + i) * R + r] = tile[threadIdx.x][i];
}

hipError_t launch_transpose(int R, int C, int act, const void *in, void *out, hipStream_t s) {
    dim3 grid((C + 31) / 32, (R + 31) / 32), block(32, 8);
    if (act == R3_BF16)
        transpose_kernel<bf16_t><<<grid, block, 0, s>>>(R, C, (const bf16_t *)in, (bf16_t *)out);
    else
        transpose_kernel<float><<<grid, block, 0, s>>>(R, C, (const float *)in, (float *)out);
    return hipGetLastError();
}

// column sums of the dense ds [T,E] -> dbias[E] (f32), fixed order: one thread
// per expert walks the tokens in ascending order in 64 interleaved partials,
// combined in a fixed tree.
template <typename T>
__global__ void __launch_bounds__(64)
colsum_kernel(int Tn, int E, const T *__restrict__ ds, float *__restrict__ out, int accumulate) {
    const int e = blockIdx.x, lane = threadIdx.x;
    const int dsw = (sizeof(T) == 2) ? 2 * E : E;
    float acc = 0.0f;
    for (int t = lane; t < Tn; t += kWave) {
        acc += Elem<T>::ld(ds + (int64_t)t * dsw + e);
        if (sizeof(T) == 2) acc += Elem<T>::ld(ds + (int64_t)t * dsw + E + e);
    }
    acc = wave_sum(acc);
    if (lane == 0) out[e] = accumulate ? out[e] + acc : acc;
}

hipError_t launch_colsum(int T, int E, int act, const void *ds, float *out, int accumulate, hipStream_t s) {
    if (act == R3_BF16)
        colsum_kernel<bf16_t><<<E, 64, 0, s>>>(T, E, (const bf16_t *)ds, out, accumulate);
    else
        colsum_kernel<float><<<E, 64, 0, s>>>(T, E, (const float *)ds, out, accumulate);
    return hipGetLastError();
}

}  // namespace r3
