// TopKMask selection shared by the record kernel and the fused router kernel: order keys and the
// 8-lanes-per-token selection of the K <= 8 largest of E = 32 NV logits (Section 4.1, second equation).
#pragma once
#include "r3_common.h"

namespace r3 {

// Order-preserving map float -> uint32 (larger float = larger key), with
// -0 == +0 and every NaN mapped to 0, below -inf.
__device__ __forceinline__ uint32_t order_key(float v, bool &nonfinite) {
    uint32_t u = __float_as_uint(v);
    uint32_t mag = u & 0x7fffffffu;
    nonfinite = mag >= 0x7f800000u;
    if (mag > 0x7f800000u) return 0u;      // NaN
    if (mag == 0u) u = 0u;                 // -0 -> +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ void cmpx_desc(uint32_t &a, uint32_t &b) {
    const uint32_t hi = max(a, b), lo = min(a, b);
    a = hi;
    b = lo;
}

// Value of lane `partner(lane)` inside each group of 8 lanes, through DPP (a VALU move, no LDS
// round trip): STEP 0: lane^1, STEP 1: lane^2 (quad permutes), STEP 2: 7 - lane%8 (half-row
// mirror).  After the three steps every lane of a group has met every other one.
template <int STEP>
__device__ __forceinline__ uint32_t group8_exchange(uint32_t v) {
    constexpr int ctrl = STEP == 0 ? 0xB1 : STEP == 1 ? 0x4E : 0x141;
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, 0xf, 0xf, false);
}

__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
    return max(min(a, b), min(max(a, b), c));
}

template <int STEP>
__device__ __forceinline__ void merge_top8(uint32_t (&top)[8]) {
    uint32_t other[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) other[j] = group8_exchange<STEP>(top[j]);
#pragma unroll
    for (int j = 0; j < 8; ++j) top[j] = max(top[j], other[7 - j]);
    cmpx_desc(top[0], top[4]); cmpx_desc(top[1], top[5]); cmpx_desc(top[2], top[6]); cmpx_desc(top[3], top[7]);
    cmpx_desc(top[0], top[2]); cmpx_desc(top[1], top[3]); cmpx_desc(top[4], top[6]); cmpx_desc(top[5], top[7]);
    cmpx_desc(top[0], top[1]); cmpx_desc(top[2], top[3]); cmpx_desc(top[4], top[5]); cmpx_desc(top[6], top[7]);
}

// The K <= 8 largest of a token's E = 32 NV keys as an E-bit mask (word i, bit b = id 32 i + b), ties to
// the lower id.  The 8 lanes of a token hold the keys of ids 32 i + 4 sub + c in key[i][c]; every lane
// of the group returns the same mask.  Each lane keeps its 8 largest keys in a sorted register list
// (insertion by median: new top[j] = med(top[j-1], top[j], v)), three butterfly merges leave every lane
// with the token's 8 largest, the K-th of them is the threshold: "above it" and "equal to it" become
// masks OR-ed over the lanes, and the equal ones are taken lowest id first until K bits are set.
template <int NV>
__device__ __forceinline__ void topk_mask8(const uint32_t (&key)[NV][4], int K, int sub, uint32_t (&gt)[NV]) {
    uint32_t top[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) top[j] = 0u;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t v = key[i][c];
            uint32_t nt[8];
            nt[0] = max(top[0], v);
#pragma unroll
            for (int j = 1; j < 8; ++j) nt[j] = umed3(top[j - 1], top[j], v);
#pragma unroll
            for (int j = 0; j < 8; ++j) top[j] = nt[j];
        }
    merge_top8<0>(top);
    merge_top8<1>(top);
    merge_top8<2>(top);
    uint32_t thr = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j == K - 1) thr = top[j];
    uint32_t eq[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        uint32_t g = 0u, q = 0u;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            g |= (uint32_t)(key[i][c] > thr) << c;
            q |= (uint32_t)(key[i][c] == thr) << c;
        }
        gt[i] = g << (4 * sub);
        eq[i] = q << (4 * sub);
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        gt[i] |= group8_exchange<0>(gt[i]);
        eq[i] |= group8_exchange<0>(eq[i]);
        gt[i] |= group8_exchange<1>(gt[i]);
        eq[i] |= group8_exchange<1>(eq[i]);
        gt[i] |= group8_exchange<2>(gt[i]);
        eq[i] |= group8_exchange<2>(eq[i]);
    }
    int quota = K;
#pragma unroll
    for (int i = 0; i < NV; ++i) quota -= __popc(gt[i]);
    // equal keys: lowest ids first, `quota` of them
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        uint32_t w = eq[i];
        const int c = __popc(w);
        if (c <= quota) {
            gt[i] |= w;
            quota -= c;
        } else {
            while (quota > 0) {
                const uint32_t b = w & (0u - w);
                gt[i] |= b;
                w ^= b;
                --quota;
            }
        }
    }
}

}  // namespace r3
