// 256x256x64 bf16 MFMA tile loop for gfx950 with direct global->LDS loads.
//
// D[p][q] = sum_k P[p][k] * Q[q][k], f32 accumulation; P feeds the MFMA A operand
// (output's contiguous dimension), Q the B operand (output rows).  8 waves, arranged
// 2 (P) x 4 (Q), each owning a 128 x 64 block as 4 x 2 MFMA 32x32x16 tiles.
//
// Operand tiles (32 KB each) are fetched with buffer_load_dwordx4 ... lds: a wave's
// 64 lanes deposit 64 x 16 B at consecutive LDS addresses, so LDS writes are
// conflict-free by construction and need no VGPR staging; the XOR swizzle that makes the
// later fragment reads conflict-free is applied on the global side (each lane fetches the
// 16-byte chunk that belongs in its LDS slot).  Buffer descriptors give bounds checking:
// rows past the end of an expert's segment read as zero, which is exactly what the ragged
// reduction of the weight gradients needs, and keeps every access in bounds.
//
// Tile forms in LDS:
//   KC   [256 rows][64 k]          row = 128 B; 16-B chunk c of row r sits at c ^ ((r>>1)&7)
//   TR   [64 k][R features]        k-row = 2R B; 64-B group g of k-row k sits at g ^ (k&3);
//        fragments come out through ds_read_b64_tr_b16 (4 consecutive k of one feature).
// Two LDS stages are separate arrays so that the compiler can see that the loads in
// flight never alias the stage being read (no vmcnt wait in front of the fragment reads).
#pragma once
#include "r3_mfma.h"

namespace r3 {

constexpr int kBK2 = 64;
constexpr int kTile = 256;
constexpr int kOperandBytes = kTile * kBK2 * 2;  // 32 KB
constexpr int kStageBytes = 2 * kOperandBytes;   // 64 KB
constexpr int kWaves2 = 8, kThreads2 = 512;
constexpr int kWP2 = 2, kWQ2 = 4, kTP2 = 4, kTQ2 = 2;
constexpr uint32_t kRsrcFlags = 0x00020000u;

typedef __attribute__((address_space(3))) void *lds_void_ptr;

// One source window: `base` points at the tile's first row/k-row (column 0 of the
// matrix), `nbytes` are the bytes from there that may be read (anything beyond reads 0),
// `step` is how far one k-tile advances.
struct Src {
    const char *base;
    uint32_t nbytes;
    uint32_t step;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t src_rsrc(const Src &s, int kt) {
    const uint64_t adv = (uint64_t)kt * s.step;
    const uint32_t left = adv < s.nbytes ? (uint32_t)(s.nbytes - adv) : 0u;
    return __builtin_amdgcn_make_buffer_rsrc((void *)(s.base + adv), (short)0, (int)left, (int)kRsrcFlags);
}

// K-contiguous 256-row tile.  ld_bytes = row pitch of the source, col_bytes = byte offset
// of k = 0 inside a source row.
struct DmaKC {
    int voff[4];
    __device__ __forceinline__ void init(int ld_bytes) {
        const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 8 * (w + kWaves2 * i) + (lane >> 3);
            const int c = (lane & 7) ^ ((row >> 1) & 7);
            voff[i] = row * ld_bytes + c * 16;
        }
    }
    __device__ __forceinline__ void issue_one(__amdgpu_buffer_rsrc_t r, char *tile, int i) const {
        const int w = threadIdx.x >> 6;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void_ptr)(tile + 1024 * (w + kWaves2 * i)), 16, voff[i],
                                                 0, 0, 0);
    }
    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t r, char *tile) const {
#pragma unroll
        for (int i = 0; i < 4; ++i) issue_one(r, tile, i);
    }
};

// Transposed tile: 64 k-rows of R features (R = 256: one tile of 32 KB; R = 128: 16 KB).
// col_bytes = byte offset of the tile's first feature inside a source row.
template <int R>
struct DmaTR {
    static constexpr int NCH = R / 8;             // 1 KB chunks in the tile
    static constexpr int PER = NCH / kWaves2;     // chunks per wave
    static constexpr int LPR = R / 8;             // lanes (16-B slots) per k-row
    static constexpr int KR = 64 / LPR;           // k-rows per chunk
    int voff[PER];
    __device__ __forceinline__ void init(int ld_bytes, int col_bytes) {
        const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int k = KR * (w + kWaves2 * i) + lane / LPR;
            const int pc = lane % LPR;
            const int c16 = (((pc >> 2) ^ (k & 3)) << 2) | (pc & 3);
            voff[i] = k * ld_bytes + col_bytes + c16 * 16;
        }
    }
    __device__ __forceinline__ void issue_one(__amdgpu_buffer_rsrc_t r, char *tile, int i) const {
        const int w = threadIdx.x >> 6;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void_ptr)(tile + 1024 * (w + kWaves2 * i)), 16, voff[i],
                                                 0, 0, 0);
    }
    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t r, char *tile) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) issue_one(r, tile, i);
    }
};

// Operand kinds.  Each provides: init, issue(kt, stage_tile), frag(stage_tile, t, s).
//   KC256  : one Src
//   TR256  : one Src
//   TR128x2: two Src (sub-tile 0 at tile+0, sub-tile 1 at tile+16 KB); MFMA tiles 0,1 of a
//            wave come from sub-tile 0 and tiles 2,3 from sub-tile 1 at the same features
// A second Src set takes over from k-tile `kswitch` on (two-phase reductions).
struct OpKC256 {
    static constexpr int kDsReads = kTP2, kDsReadsQ = kTQ2;  // ds_read_b128 per sub-step as P / as Q
    Src src[2];
    int kswitch;
    DmaKC dma;
    KcFrag<kBK2> fr;
    __device__ __forceinline__ void init(int ld_bytes, int wave_base) {
        dma.init(ld_bytes);
        fr.init(wave_base);
    }
    __device__ __forceinline__ void issue(int kt, char *tile) const {
        const bool second = kt >= kswitch;
        const Src &s = second ? src[1] : src[0];
        dma.issue(src_rsrc(s, second ? kt - kswitch : kt), tile);
    }
    // one quarter (part = 0..3) of the tile's loads
    __device__ __forceinline__ void issue_part(int kt, char *tile, int part) const {
        const bool second = kt >= kswitch;
        const Src &s = second ? src[1] : src[0];
        dma.issue_one(src_rsrc(s, second ? kt - kswitch : kt), tile, part);
    }
    __device__ __forceinline__ bf16x8_t frag(const char *tile, int t, int s) const { return fr.read(tile, t, s); }
};

struct OpTR256 {
    static constexpr int kDsReads = 2 * kTP2, kDsReadsQ = 2 * kTQ2;  // two ds_read_b64_tr_b16 per fragment
    Src src[2];
    int kswitch;
    DmaTR<256> dma;
    TrFrag<256> fr;
    __device__ __forceinline__ void init(int ld_bytes, int col_bytes, int wave_base) {
        dma.init(ld_bytes, col_bytes);
        fr.init(wave_base);
    }
    __device__ __forceinline__ void issue(int kt, char *tile) const {
        const bool second = kt >= kswitch;
        const Src &s = second ? src[1] : src[0];
        dma.issue(src_rsrc(s, second ? kt - kswitch : kt), tile);
    }
    __device__ __forceinline__ void issue_part(int kt, char *tile, int part) const {
        const bool second = kt >= kswitch;
        const Src &s = second ? src[1] : src[0];
        dma.issue_one(src_rsrc(s, second ? kt - kswitch : kt), tile, part);
    }
    __device__ __forceinline__ bf16x8_t frag(const char *tile, int t, int s) const { return fr.read(tile, t, s); }
};

struct OpTR128x2 {
    static constexpr int kDsReads = 2 * kTP2, kDsReadsQ = 2 * kTQ2;
    Src src[2];  // sub-tile 0, sub-tile 1
    DmaTR<128> dma;
    TrFrag<128> fr;
    __device__ __forceinline__ void init(int ld_bytes, int col_bytes, int wave_base) {
        dma.init(ld_bytes, col_bytes);
        fr.init(wave_base);
    }
    __device__ __forceinline__ void issue(int kt, char *tile) const {
        dma.issue(src_rsrc(src[0], kt), tile);
        dma.issue(src_rsrc(src[1], kt), tile + kOperandBytes / 2);
    }
    __device__ __forceinline__ void issue_part(int kt, char *tile, int part) const {
        dma.issue_one(src_rsrc(src[part >> 1], kt), tile + (part >> 1) * (kOperandBytes / 2), part & 1);
    }
    __device__ __forceinline__ bf16x8_t frag(const char *tile, int t, int s) const {
        return fr.read(tile + (t >> 1) * (kOperandBytes / 2), t & 1, s);
    }
};

typedef f32x16_t Acc2[kTP2][kTQ2];

__device__ __forceinline__ void zero_acc2(Acc2 &acc) {
#pragma unroll
    for (int i = 0; i < kTP2; ++i)
#pragma unroll
        for (int j = 0; j < kTQ2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
}

struct Frags {
    bf16x8_t a[kTP2], b[kTQ2];
};

template <class POp, class QOp>
__device__ __forceinline__ void read_frags(Frags &f, const POp &P, const QOp &Q, const char *stage, int s) {
#pragma unroll
    for (int i = 0; i < kTP2; ++i) f.a[i] = P.frag(stage, i, s);
#pragma unroll
    for (int j = 0; j < kTQ2; ++j) f.b[j] = Q.frag(stage + kOperandBytes, j, s);
}

__device__ __forceinline__ void mfma_block(Acc2 &acc, const Frags &f) {
#pragma unroll
    for (int i = 0; i < kTP2; ++i)
#pragma unroll
        for (int j = 0; j < kTQ2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
}

// One resident stage.  On entry `x` may hold the last fragment set of the previous stage
// (pending = true): its MFMAs are issued right after this stage's first fragment reads, so
// the MFMA pipe has work while those reads are in flight just after the barrier.  On exit
// `x` holds this stage's last fragment set, not yet multiplied.
// The sched_barriers keep at most two fragment sets live next to the 128 accumulators.
// One sub-step: the fragment reads of the next 16 k go out first, then (first sub-step only)
// the next stage's global->LDS loads, then the 8 MFMAs of the current fragments, so the reads
// have 8 MFMAs (256 cycles) to land.  (Left alone the compiler sinks the reads below the
// MFMAs and every sub-step starts by waiting on LDS.  Spreading the loads over the four
// sub-steps was measured slower: the late ones are not back before the stage ends.)
template <class POp, class QOp>
__device__ __forceinline__ void sub_step(Acc2 &acc, Frags &next, const Frags &cur, const POp &P, const QOp &Q,
                                         const char *stage, int s, bool prefetch, int kt_next, char *stage_next) {
    read_frags(next, P, Q, stage, s);
    if (prefetch && s == 0) {
        P.issue(kt_next, stage_next);
        Q.issue(kt_next, stage_next + kOperandBytes);
    }
    mfma_block(acc, cur);
    __builtin_amdgcn_sched_group_barrier(0x100, POp::kDsReads + QOp::kDsReadsQ, 0);  // DS reads
    if (s == 0) __builtin_amdgcn_sched_group_barrier(0x020, 8, 0);                   // VMEM reads
    __builtin_amdgcn_sched_group_barrier(0x008, kTP2 * kTQ2, 0);                     // MFMA
    __builtin_amdgcn_sched_barrier(0);
}

// One resident stage.  On entry `x` holds the last fragment set of the previous stage (zeros
// on the very first stage): its MFMAs are issued right behind this stage's first fragment
// reads, so the MFMA pipe has work while those reads are in flight just after the barrier.
// On exit `x` holds this stage's last fragment set, not yet multiplied.  At most two fragment
// sets are live next to the 128 accumulator registers.
template <class POp, class QOp>
__device__ __forceinline__ void stage_compute(Acc2 &acc, Frags &x, Frags &y, const POp &P, const QOp &Q,
                                              const char *stage, bool prefetch, int kt_next, char *stage_next) {
    sub_step(acc, y, x, P, Q, stage, 0, prefetch, kt_next, stage_next);
    sub_step(acc, x, y, P, Q, stage, 1, prefetch, kt_next, stage_next);
    sub_step(acc, y, x, P, Q, stage, 2, prefetch, kt_next, stage_next);
    sub_step(acc, x, y, P, Q, stage, 3, prefetch, kt_next, stage_next);
}

// nk k-tiles of 64.  s0, s1: the two 64 KB LDS stages (distinct arrays).
template <class POp, class QOp>
__device__ __forceinline__ void mfma_mainloop2(Acc2 &acc, int nk, const POp &P, const QOp &Q, char *s0, char *s1) {
    if (nk <= 0) return;
    P.issue(0, s0);
    Q.issue(0, s0 + kOperandBytes);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    Frags x, y;
#pragma unroll
    for (int i = 0; i < kTP2; ++i) x.a[i] = bf16x8_t{};
#pragma unroll
    for (int j = 0; j < kTQ2; ++j) x.b[j] = bf16x8_t{};
    for (int kt = 0; kt < nk; kt += 2) {
        const bool has1 = kt + 1 < nk, has2 = kt + 2 < nk;
        stage_compute(acc, x, y, P, Q, s0, has1, kt + 1, s1);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        // single loop exit (no break) keeps the accumulators in place
        if (has1) stage_compute(acc, x, y, P, Q, s1, has2, kt + 2, s0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }
    mfma_block(acc, x);
}

// Visit the wave's results as groups of 4 consecutive p for one q (tile-local p, q).
template <class F>
__device__ __forceinline__ void for_each_quad2(F f) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wp = wave % kWP2, wq = wave / kWP2;
#pragma unroll
    for (int tp = 0; tp < kTP2; ++tp)
#pragma unroll
        for (int tq = 0; tq < kTQ2; ++tq)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                f(tp, tq, g, wp * 128 + tp * 32 + g * 8 + (lane >> 5) * 4, wq * 64 + tq * 32 + (lane & 31));
}

__device__ __forceinline__ uint32_t clamp_bytes(int64_t b) {
    return b <= 0 ? 0u : (b > 0x7fffffffLL ? 0x7fffffffu : (uint32_t)b);
}

}  // namespace r3
