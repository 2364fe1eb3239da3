// bf16 MFMA contraction core for gfx950 (CDNA4), used by every dense step of the
// replayed MoE layer: D[p][q] = sum_k P[p][k] * Q[q][k], f32 accumulation.
//
// Roles.  "P" feeds the MFMA A operand and runs along the output's contiguous
// dimension (features), "Q" feeds the B operand and runs along output rows, so
// a lane ends up with 4 consecutive features of one row and stores 8 (bf16) or
// 16 (f32) contiguous bytes.
//
// Each operand tile is staged in LDS in one of two forms:
//   KC  rows of BK contiguous k (source matrix is [row][k]); fragments are read
//       with 16-byte ds_read_b128.
//   TR  BK rows of R contiguous features (source matrix is [k][feature]);
//       fragments are read with the gfx950 transposing read ds_read_b64_tr_b16,
//       which hands each lane 4 consecutive k of one feature.
// Both forms are XOR-swizzled for the 64-bank LDS so that reads and writes are
// conflict-free without padding.  LDS is double-buffered: global loads for tile
// kt+1 are issued before the MFMAs of tile kt and written to the other buffer
// after them, one barrier per k-tile.
#pragma once
#include "r3_common.h"

namespace r3 {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;

// BP x BQ output tile, WP x WQ waves, BK k per stage.
template <int BP_, int BQ_, int WP_, int WQ_, int BK_>
struct TileCfg {
    static constexpr int BP = BP_, BQ = BQ_, WP = WP_, WQ = WQ_, BK = BK_;
    static constexpr int NWAVES = WP * WQ, NT = 64 * NWAVES;
    static constexpr int WTP = BP / WP, WTQ = BQ / WQ;  // wave tile
    static constexpr int TP = WTP / 32, TQ = WTQ / 32;  // 32x32 MFMA tiles per wave
    static constexpr int P_BYTES = BP * BK * 2, Q_BYTES = BQ * BK * 2;
    static constexpr int STAGE = P_BYTES + Q_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE;
    static constexpr int CH = BK / 8;                    // 16-byte chunks per KC row
    static constexpr int NP = BP * CH / NT, NQ = BQ * CH / NT;  // chunks per thread
    static_assert(WTP % 32 == 0 && WTQ % 32 == 0, "wave tile must be a multiple of 32");
    static_assert((BP * CH) % NT == 0 && (BQ * CH) % NT == 0, "tile/threads mismatch");
    static_assert(BK == 32 || BK == 64, "BK");
};

// byte offset of 16-byte chunk c of row `row` in a KC tile (row = BK bf16)
template <int BK>
__device__ __forceinline__ int kc_off(int row, int c) {
    constexpr int CH = BK / 8;         // chunks per row
    constexpr int RPL = 16 / CH;       // rows per 256-byte bank line
    return row * (BK * 2) + ((c ^ ((row / RPL) & (CH - 1))) << 4);
}
// byte offset of 16-byte chunk c16 of k-row `k` in a TR tile with R features
template <int R>
__device__ __forceinline__ int tr_off(int k, int c16) {
    static_assert(R >= 128, "TR tiles need at least 128 features");
    return k * (R * 2) + (((((c16 >> 2) ^ (k & 3)) << 2) | (c16 & 3)) << 4);
}

// Fragment readers: return the 8 consecutive-k bf16 values of MFMA row/col
// (lane & 31) for k-group (lane >> 5) of 16-wide k step `s`, sub-tile ti.
template <int BK>
struct KcFrag {
    int base;  // per-lane byte offset without the chunk term
    int swz;
    int hi;
    __device__ __forceinline__ void init(int wave_base, int lane = lane_id()) {
        const int row = wave_base + (lane & 31);
        constexpr int CH = BK / 8, RPL = 16 / CH;
        base = row * (BK * 2);
        swz = (row / RPL) & (CH - 1);
        hi = lane >> 5;
    }
    __device__ __forceinline__ bf16x8_t read(const char *tile, int ti, int s) const {
        const int off = base + ti * 32 * (BK * 2) + (((2 * s + hi) ^ swz) << 4);
        return *(const bf16x8_t *)(tile + off);
    }
};

template <int R>
struct TrFrag {
    int lane_off;  // k-row and sub-chunk part
    int kx;        // k & 3 of this lane's rows
    int cbase;     // c16 of the wave's first feature
    int clo;       // c16 & 3 part that depends on the lane
    __device__ __forceinline__ void init(int wave_base) {
        const int lane = lane_id();
        const int b = lane >> 4, i = lane & 15;
        kx = (i >> 2) & 3;
        lane_off = (8 * (b >> 1) + (i >> 2)) * (R * 2) + (i & 1) * 8;
        cbase = wave_base >> 3;
        clo = 2 * (b & 1) + ((i & 3) >> 1);
    }
    __device__ __forceinline__ bf16x8_t read(const char *tile, int ti, int s) const {
        const int c16 = cbase + 4 * ti + clo;
        const int col = ((((c16 >> 2) ^ kx) << 2) | (c16 & 3)) << 4;
        const char *p = tile + lane_off + col + s * 16 * (R * 2);
        s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
        s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * (R * 2)));
        s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8_t, v);
    }
};

template <bool TRANSPOSED, int R, int BK> struct FragSel { typedef KcFrag<BK> type; };
template <int R, int BK> struct FragSel<true, R, BK> { typedef TrFrag<R> type; };

// Main loop.  fp(kt, i, c) / fq(kt, i, c) return the 16-byte chunk of k-tile kt:
//   KC operand: i = row in tile, c = chunk along k (8 bf16 each)
//   TR operand: i = k row in tile, c = chunk along features
// acc[tp][tq] is the 32x32 block (tp along P, tq along Q) of the wave's tile.
template <class TL, bool PTR, bool QTR, class FP, class FQ>
__device__ __forceinline__ void mfma_mainloop(f32x16_t (&acc)[TL::TP][TL::TQ], int nk, FP fp, FQ fq,
                                              char *lds) {
    constexpr int BK = TL::BK, NT = TL::NT;
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int wp = wave % TL::WP, wq = wave / TL::WP;

    uint4 rp[TL::NP], rq[TL::NQ];

    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < TL::NP; ++i) {
            const int id = tid + i * NT;
            if constexpr (PTR) rp[i] = fp(kt, id / (TL::BP / 8), id % (TL::BP / 8));
            else rp[i] = fp(kt, id / TL::CH, id % TL::CH);
        }
#pragma unroll
        for (int i = 0; i < TL::NQ; ++i) {
            const int id = tid + i * NT;
            if constexpr (QTR) rq[i] = fq(kt, id / (TL::BQ / 8), id % (TL::BQ / 8));
            else rq[i] = fq(kt, id / TL::CH, id % TL::CH);
        }
    };
    auto lstore = [&](int stage) {
        char *pb = lds + stage * TL::STAGE;
        char *qb = pb + TL::P_BYTES;
#pragma unroll
        for (int i = 0; i < TL::NP; ++i) {
            const int id = tid + i * NT;
            int off;
            if constexpr (PTR) off = tr_off<TL::BP>(id / (TL::BP / 8), id % (TL::BP / 8));
            else off = kc_off<BK>(id / TL::CH, id % TL::CH);
            *(uint4 *)(pb + off) = rp[i];
        }
#pragma unroll
        for (int i = 0; i < TL::NQ; ++i) {
            const int id = tid + i * NT;
            int off;
            if constexpr (QTR) off = tr_off<TL::BQ>(id / (TL::BQ / 8), id % (TL::BQ / 8));
            else off = kc_off<BK>(id / TL::CH, id % TL::CH);
            *(uint4 *)(qb + off) = rq[i];
        }
    };

    typename FragSel<PTR, TL::BP, BK>::type pf;
    typename FragSel<QTR, TL::BQ, BK>::type qf;
    pf.init(wp * TL::WTP);
    qf.init(wq * TL::WTQ);

    if (nk <= 0) return;
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) gload(kt + 1);
        const char *pb = lds + (kt & 1) * TL::STAGE;
        const char *qb = pb + TL::P_BYTES;
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            bf16x8_t a[TL::TP], b[TL::TQ];
#pragma unroll
            for (int i = 0; i < TL::TP; ++i) a[i] = pf.read(pb, i, s);
#pragma unroll
            for (int j = 0; j < TL::TQ; ++j) b[j] = qf.read(qb, j, s);
#pragma unroll
            for (int i = 0; i < TL::TP; ++i)
#pragma unroll
                for (int j = 0; j < TL::TQ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) lstore((kt + 1) & 1);
        __syncthreads();
    }
}

// The same loop with the global loads running two k-tiles ahead (two register sets): for skinny
// contractions that are bound by memory latency, not arithmetic (the router: one token tile per
// work-group, 32 k-tiles in a row, each otherwise waiting a full round trip for its loads).
// While tile kt is multiplied, tile kt+1 is on its way into registers (asked for an iteration ago)
// and tile kt+2 is asked for; tile kt+1 goes to the other LDS stage after the multiplication.
template <class TL, bool PTR, bool QTR, class FP, class FQ>
__device__ __forceinline__ void mfma_mainloop_ahead2(f32x16_t (&acc)[TL::TP][TL::TQ], int nk, FP fp, FQ fq,
                                                     char *lds) {
    constexpr int BK = TL::BK, NT = TL::NT;
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int wp = wave % TL::WP, wq = wave / TL::WP;
    uint4 rp[2][TL::NP], rq[2][TL::NQ];
    auto gload = [&](int kt, uint4 (&p)[TL::NP], uint4 (&q)[TL::NQ]) {
#pragma unroll
        for (int i = 0; i < TL::NP; ++i) {
            const int id = tid + i * NT;
            if constexpr (PTR) p[i] = fp(kt, id / (TL::BP / 8), id % (TL::BP / 8));
            else p[i] = fp(kt, id / TL::CH, id % TL::CH);
        }
#pragma unroll
        for (int i = 0; i < TL::NQ; ++i) {
            const int id = tid + i * NT;
            if constexpr (QTR) q[i] = fq(kt, id / (TL::BQ / 8), id % (TL::BQ / 8));
            else q[i] = fq(kt, id / TL::CH, id % TL::CH);
        }
    };
    auto lstore = [&](int stage, const uint4 (&p)[TL::NP], const uint4 (&q)[TL::NQ]) {
        char *pb = lds + stage * TL::STAGE;
        char *qb = pb + TL::P_BYTES;
#pragma unroll
        for (int i = 0; i < TL::NP; ++i) {
            const int id = tid + i * NT;
            int off;
            if constexpr (PTR) off = tr_off<TL::BP>(id / (TL::BP / 8), id % (TL::BP / 8));
            else off = kc_off<BK>(id / TL::CH, id % TL::CH);
            *(uint4 *)(pb + off) = p[i];
        }
#pragma unroll
        for (int i = 0; i < TL::NQ; ++i) {
            const int id = tid + i * NT;
            int off;
            if constexpr (QTR) off = tr_off<TL::BQ>(id / (TL::BQ / 8), id % (TL::BQ / 8));
            else off = kc_off<BK>(id / TL::CH, id % TL::CH);
            *(uint4 *)(qb + off) = q[i];
        }
    };
    typename FragSel<PTR, TL::BP, BK>::type pf;
    typename FragSel<QTR, TL::BQ, BK>::type qf;
    pf.init(wp * TL::WTP);
    qf.init(wq * TL::WTQ);
    auto multiply = [&](int stage) {
        const char *pb = lds + stage * TL::STAGE;
        const char *qb = pb + TL::P_BYTES;
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            bf16x8_t a[TL::TP], b[TL::TQ];
#pragma unroll
            for (int i = 0; i < TL::TP; ++i) a[i] = pf.read(pb, i, s);
#pragma unroll
            for (int j = 0; j < TL::TQ; ++j) b[j] = qf.read(qb, j, s);
#pragma unroll
            for (int i = 0; i < TL::TP; ++i)
#pragma unroll
                for (int j = 0; j < TL::TQ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };
    if (nk <= 0) return;
    gload(0, rp[0], rq[0]);
    if (nk > 1) gload(1, rp[1], rq[1]);
    lstore(0, rp[0], rq[0]);
    __syncthreads();
    // tile kt sits in stage kt & 1 and came through register set kt & 1; unrolled by two so that both
    // are compile-time constants
    for (int kt = 0; kt < nk; kt += 2) {
        if (kt + 2 < nk) gload(kt + 2, rp[0], rq[0]);
        multiply(0);
        if (kt + 1 < nk) lstore(1, rp[1], rq[1]);
        __syncthreads();
        if (kt + 1 < nk) {
            if (kt + 3 < nk) gload(kt + 3, rp[1], rq[1]);
            multiply(1);
            if (kt + 2 < nk) lstore(0, rp[0], rq[0]);
            __syncthreads();
        }
    }
}

template <class TL>
__device__ __forceinline__ void zero_acc(f32x16_t (&acc)[TL::TP][TL::TQ]) {
#pragma unroll
    for (int i = 0; i < TL::TP; ++i)
#pragma unroll
        for (int j = 0; j < TL::TQ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
}

// Visit the wave's results as groups of 4 consecutive p for one q:
//   f(tp, tq, g, p, q) where p, q are tile-local and acc[tp][tq][4g..4g+3] are the values.
template <class TL, class F>
__device__ __forceinline__ void for_each_quad(F f) {
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int wp = wave % TL::WP, wq = wave / TL::WP;
#pragma unroll
    for (int tp = 0; tp < TL::TP; ++tp)
#pragma unroll
        for (int tq = 0; tq < TL::TQ; ++tq)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int p = wp * TL::WTP + tp * 32 + g * 8 + (lane >> 5) * 4;
                const int q = wq * TL::WTQ + tq * 32 + (lane & 31);
                f(tp, tq, g, p, q);
            }
}

// XCD-aware work-group -> logical tile id.  Work-groups are handed to the 8 XCDs
// round-robin; giving each XCD one contiguous range of the tile list keeps the
// tiles that share an expert's weights inside one L2.  Returns -1 when idle.
__device__ __forceinline__ int xcd_tile_id(int total) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per = (total + 7) >> 3;
    const int id = xcd * per + slot;
    return (slot < per && id < total) ? id : -1;
}

__device__ __forceinline__ uint4 ld16(const bf16_t *p) { return *(const uint4 *)p; }
__device__ __forceinline__ uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }

}  // namespace r3
