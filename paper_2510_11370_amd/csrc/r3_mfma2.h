// 256x256 bf16 MFMA tile loops for gfx950 with direct global->LDS loads: a ring of 32-k stages
// (loads issued two stages ahead; used where both operands are transposed tiles) and, further
// down, a two-buffer loop over 64-k windows (used where an operand is K-contiguous).
//
// D[p][q] = sum_k P[p][k] * Q[q][k], f32 accumulation; P feeds the MFMA A operand
// (output's contiguous dimension), Q the B operand (output rows).  8 waves, arranged
// 2 (P) x 4 (Q), each owning a 128 x 64 block as 4 x 2 MFMA 32x32x16 tiles.
//
// Operand tiles (16 KB each per stage) are fetched with buffer_load_dwordx4 ... lds: a
// wave's 64 lanes deposit 64 x 16 B at consecutive LDS addresses, so LDS writes are
// conflict-free by construction and need no VGPR staging; the XOR swizzle that makes the
// later fragment reads conflict-free is applied on the global side (each lane fetches the
// 16-byte chunk that belongs in its LDS slot).  Buffer descriptors give bounds checking:
// rows past the end of an expert's segment read as zero, which is exactly what the ragged
// reduction of the weight gradients needs, and keeps every access in bounds.
//
// Tile forms in LDS (per stage):
//   KC   [256 rows][32 k]     row = 64 B; 16-B chunk c of row r sits at c ^ ((r>>2)&3)
//   TR   [32 k][R features]   k-row = 2R B; 64-B group g of k-row k sits at g ^ (k&3);
//        fragments come out through ds_read_b64_tr_b16 (4 consecutive k of one feature).
// The four stages are separate LDS arrays so that the compiler can see that loads in
// flight never alias the stage being read (no vmcnt wait in front of the fragment reads).
// Wave roles.  All 8 waves multiply.  Waves 0-3 ("loaders") also issue every tile load and
// count them: each issues the same number of loads per stage (a stage past the end of the
// reduction gets a zero-length descriptor), so "s_waitcnt vmcnt(one stage's worth)" at the end
// of stage kt is exactly "stage kt+1 has landed" (a third stage of prefetch was measured: no gain).  (Having waves 4-7 touch the lines of
// later stages to warm L2 was tried and measured slower: the extra requests cost more in the
// vector memory path than the shorter load latency gave back.)
#pragma once
#include "r3_mfma.h"

namespace r3 {

constexpr int kBK2 = 32;
constexpr int kTile = 256;
constexpr int kStages2 = 4;
constexpr int kOperandBytes = kTile * kBK2 * 2;  // 16 KB
constexpr int kStageBytes = 2 * kOperandBytes;   // 32 KB
#ifndef R3_GEMM_WAVES
#define R3_GEMM_WAVES 8
#endif
#if R3_GEMM_WAVES == 8
// 2 (P) x 4 (Q) waves of 128 x 64, two per SIMD; waves 0-3 also load
constexpr int kWaves2 = 8, kThreads2 = 512, kMinWavesPerSimd = 2;
constexpr int kWP2 = 2, kWQ2 = 4, kTP2 = 4, kTQ2 = 2;
constexpr int kReadsPerMfma = 2;   // fragment reads threaded behind each MFMA of a sub-step
#else
// 2 x 2 waves of 128 x 128, one per SIMD (accumulators in the second half of the 512
// registers a lone wave may use); every wave loads.  A third less LDS read traffic, but
// measured 5 % (weight gradients) to 30 % (kernels with wide epilogues) slower than the
// 8-wave form on the 16384-token layer: a lone wave has nobody to cover its stalls.
constexpr int kWaves2 = 4, kThreads2 = 256, kMinWavesPerSimd = 1;
constexpr int kWP2 = 2, kWQ2 = 2, kTP2 = 4, kTQ2 = 4;
constexpr int kReadsPerMfma = 1;
#endif
constexpr int kLoaderWaves = 4;
constexpr int kWaveRowsQ = 32 * kTQ2;            // output rows (Q) per wave
constexpr uint32_t kRsrcFlags = 0x00020000u;

typedef __attribute__((address_space(3))) void *lds_void_ptr;

// One source window: `base` points at the tile's first row/k-row (column 0 of the
// matrix), `nbytes` are the bytes from there that may be read (anything beyond reads 0),
// `step` is how far one k-tile advances.
struct Src {
    const char *base;
    uint64_t nbytes;   // a segment may exceed 4 GB; each descriptor sees at most 2 GB of what is left
    uint32_t step;
};

typedef int rsrc_t __attribute__((ext_vector_type(4)));  // buffer descriptor words (wave-uniform)

// `extra`: a further wave-uniform byte advance (the window then starts that much later and is that
// much shorter, so the bounds check stays exact)
__device__ __forceinline__ rsrc_t src_rsrc(const Src &s, int kt, uint32_t extra = 0u) {
    const uint64_t adv = (uint64_t)kt * s.step + extra;
    const uint64_t rest = adv < s.nbytes ? s.nbytes - adv : 0u;
    const uint32_t left = rest > 0x7fffffffu ? 0x7fffffffu : (uint32_t)rest;
    const uint64_t b = (uint64_t)(s.base + adv);
    // the words are wave-uniform by construction; readfirstlane makes that visible to the
    // compiler so that they live in SGPRs
    rsrc_t r = {__builtin_amdgcn_readfirstlane((int)(uint32_t)b),
                __builtin_amdgcn_readfirstlane((int)((uint32_t)(b >> 32) & 0xffffu)),
                __builtin_amdgcn_readfirstlane((int)left), (int)kRsrcFlags};
    return r;
}

// LDS byte address of a __shared__ object (the low half of its generic address)
__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)(uintptr_t)(lds_void_ptr)p; }

// buffer_load_dwordx4 ... lds: lane i's 16 bytes go to LDS address dst_wave + 16 i.
// Written as inline asm on purpose: the compiler then neither tracks these loads nor puts
// conservative vmcnt waits in front of later LDS reads (it cannot tell that a read of the
// resident stage does not alias a load two stages ahead); stage_barrier() does the
// counting.  No other instruction in these kernels uses M0.
__device__ __forceinline__ void lds_load16(rsrc_t r, uint32_t dst_wave, int voff) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst_wave);
    // (no cache hint: marked non-temporal these loads ran the row-tiled kernels at half speed --
    // the operand tiles live on being shared through L2 by the compute units of an XCD)
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(m0v), "v"(voff), "s"(r)
                 : "memory");
}

// The same with a wave-uniform byte offset in an SGPR added to the address.  The hardware's bounds
// check does not see that offset: only for windows that lie inside their buffer whatever the lane
// offsets are (weight panels: a tile's 256 rows always exist).
__device__ __forceinline__ void lds_load16_soff(rsrc_t r, uint32_t dst_wave, int voff, int soff) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst_wave);
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(m0v), "v"(voff), "s"(r),
                 "s"(__builtin_amdgcn_readfirstlane(soff))
                 : "memory");
}

// K-contiguous 256-row tile: 16 chunks of 1 KB (16 rows x 64 B), four per loader wave.
struct DmaKC {
    int voff[4];
    __device__ __forceinline__ void init(int ld_bytes) {
        const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 16 * ((w & 3) + kLoaderWaves * i) + (lane >> 2);
            const int c = (lane & 3) ^ ((row >> 2) & 3);
            voff[i] = row * ld_bytes + c * 16;
        }
    }
    __device__ __forceinline__ void issue(rsrc_t r, uint32_t tile) const {
        const int w = threadIdx.x >> 6;
#pragma unroll
        for (int i = 0; i < 4; ++i) lds_load16(r, tile + 1024 * ((w & 3) + kLoaderWaves * i), voff[i]);
    }
};

// Transposed tile: 32 k-rows of R features.  R = 256: 16 chunks (2 k-rows each), two per
// wave.  R = 128: 8 chunks (4 k-rows each), one per wave.
template <int R>
struct DmaTR {
    static constexpr int NCH = R / 16;            // 1 KB chunks in the tile
    static constexpr int PER = NCH / kLoaderWaves;  // chunks per loader wave
    static constexpr int LPR = R / 8;             // lanes (16-B slots) per k-row
    static constexpr int KR = 64 / LPR;           // k-rows per chunk
    int voff[PER];
    __device__ __forceinline__ void init(int ld_bytes, int col_bytes) {
        const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int k = KR * ((w & 3) + kLoaderWaves * i) + lane / LPR;
            const int pc = lane % LPR;
            const int c16 = (((pc >> 2) ^ (k & 3)) << 2) | (pc & 3);
            voff[i] = k * ld_bytes + col_bytes + c16 * 16;
        }
    }
    __device__ __forceinline__ void issue(rsrc_t r, uint32_t tile) const {
        const int w = threadIdx.x >> 6;
#pragma unroll
        for (int i = 0; i < PER; ++i) lds_load16(r, tile + 1024 * ((w & 3) + kLoaderWaves * i), voff[i]);
    }
};

// Operand kinds.  Each provides: init, issue(kt, stage_tile), frag(stage_tile, t, s) and
// issues exactly four loads per loader wave per stage.
//   KC256  : one Src
//   TR256  : one Src
//   TR128x2: two Src (sub-tile 0 at tile+0, sub-tile 1 at tile+8 KB); MFMA tiles 0,1 of a
//            wave come from sub-tile 0 and tiles 2,3 from sub-tile 1 at the same features
// A second Src set takes over from k-tile `kswitch` on (two-phase reductions).
struct OpKC256 {
    static constexpr bool kIndexed = false, kWindowed = false;
    static constexpr int kLoads = 4;
    static constexpr int kDsReads = kTP2, kDsReadsQ = kTQ2;  // ds_read_b128 per sub-step as P / as Q
    Src src[2];
    int kswitch;
    DmaKC dma;
    KcFrag<kBK2> fr;
    __device__ __forceinline__ void init(int ld_bytes, int wave_base) {
        dma.init(ld_bytes);
        fr.init(wave_base);
    }
    __device__ __forceinline__ void issue(int kt, uint32_t tile) const {
        const bool second = kt >= kswitch;
        const Src &s = second ? src[1] : src[0];
        dma.issue(src_rsrc(s, second ? kt - kswitch : kt), tile);
    }
    __device__ __forceinline__ bf16x8_t frag(const char *tile, int t, int s) const { return fr.read(tile, t, s); }
};

struct OpTR256 {
    static constexpr bool kIndexed = false, kWindowed = false;
    static constexpr int kLoads = 4;
    static constexpr int kDsReads = 2 * kTP2, kDsReadsQ = 2 * kTQ2;  // two ds_read_b64_tr_b16 per fragment
    Src src[2];
    int kswitch;
    DmaTR<256> dma;
    TrFrag<256> fr;
    __device__ __forceinline__ void init(int ld_bytes, int col_bytes, int wave_base) {
        dma.init(ld_bytes, col_bytes);
        fr.init(wave_base);
    }
    __device__ __forceinline__ void issue(int kt, uint32_t tile) const {
        const bool second = kt >= kswitch;
        const Src &s = second ? src[1] : src[0];
        dma.issue(src_rsrc(s, second ? kt - kswitch : kt), tile);
    }
    __device__ __forceinline__ bf16x8_t frag(const char *tile, int t, int s) const { return fr.read(tile, t, s); }
};

struct OpTR128x2 {
    static constexpr bool kIndexed = false, kWindowed = false;
    static constexpr int kLoads = 4;
    static constexpr int kDsReads = 2 * kTP2, kDsReadsQ = 2 * kTQ2;
    Src src[2];  // sub-tile 0, sub-tile 1
    DmaTR<128> dma;
    TrFrag<128> fr;
    __device__ __forceinline__ void init(int ld_bytes, int col_bytes, int wave_base) {
        dma.init(ld_bytes, col_bytes);
        fr.init(wave_base);
    }
    __device__ __forceinline__ void issue(int kt, uint32_t tile) const {
        dma.issue(src_rsrc(src[0], kt), tile);
        dma.issue(src_rsrc(src[1], kt), tile + kOperandBytes / 2);
    }
    __device__ __forceinline__ bf16x8_t frag(const char *tile, int t, int s) const {
        return fr.read(tile + (t >> 1) * (kOperandBytes / 2), t & 1, s);
    }
};

// Transposed 256-feature tile whose k-rows are gathered through an index: k-row r of the reduction is
// row rows[r] of a row-major matrix of `ld_bytes` per row, so a permuted copy of that matrix never has
// to exist.  A chunk of the tile is two k-rows, and a loader wave owns four chunks of a stage, i.e. eight
// consecutive entries of the index list.  Those eight entries travel like the tiles do: two stages
// ahead of the tile loads that use them, one more buffer load per loader wave per stage brings them
// straight into a small LDS ring of the wave's own (counted by the same vector-memory counter that
// paces the stages, so they have landed when the stage barrier lets the wave go on); the wave reads
// its four entries back with one LDS read and each lane builds its own row address.  (With scalar
// loads instead the compiler waits for them right where they are issued, every stage: measured 19 %
// on the long reductions of a skewed batch.)  Only the first two stages of a tile, which nothing ran
// ahead of, take their entries with scalar loads.  k-rows >= n read as zero (an offset outside the
// buffer window).  `rows` must be readable up to index n + 7.
typedef const __attribute__((address_space(4))) int32_t *const_i32_ptr;
constexpr int kIndexRingBytes = kLoaderWaves * 4 * 256;  // per loader wave: four slots of one 64-lane dword load
struct OpTR256G {
    static constexpr int kDsReads = 2 * kTP2, kDsReadsQ = 2 * kTQ2;
    static constexpr bool kIndexed = true, kWindowed = false;
    static constexpr int kLoads = 5;             // four tile loads and one index load
    static constexpr int kOutside = 0x7ffffff0;  // beyond any window (windows are < 2^31 bytes)
    rsrc_t rs, rsi;        // the matrix; the tile's index list
    const_i32_ptr rows;
    int n, ld_bytes, wl;
    uint32_t ring;         // LDS address of this wave's ring
    int cvoff[4];
    TrFrag<256> fr;
    __device__ __forceinline__ void init(int ld_bytes_, int wave_base, const void *ring_base) {
        wl = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6) & 3);
        ring = __builtin_amdgcn_readfirstlane((int)(lds_addr(ring_base) + 1024u * wl));
        ld_bytes = ld_bytes_;
        fr.init(wave_base);
    }
    // point at a tile: the whole matrix (`bytes` < 2^31), feature offset col_bytes, index list, live k-rows
    __device__ __forceinline__ void aim(const void *matrix, uint64_t bytes, int col_bytes, const int32_t *rows_, int n_) {
        rs = src_rsrc(Src{(const char *)matrix, bytes, 0u}, 0);
        n = __builtin_amdgcn_readfirstlane(n_);
        rsi = src_rsrc(Src{(const char *)rows_, (uint64_t)(n + 8) * 4u, 0u}, 0);
        // wave-uniform by construction (a tile's coordinates); said so, so that the first stages'
        // index fetches are scalar loads
        const uint64_t ra = (uint64_t)rows_;
        rows = (const_i32_ptr)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(ra >> 32)) << 32) |
                               (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)ra));
        col_bytes = __builtin_amdgcn_readfirstlane(col_bytes);
        const int lane = threadIdx.x & 63, pc = lane & 31;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = 2 * i + (lane >> 5);   // k-row within the wave's eight; 8 wl does not change k & 3
            cvoff[i] = col_bytes + ((((pc >> 2) ^ (k & 3)) << 2) | (pc & 3)) * 16;
        }
    }
    // The wave's eight entries of stage kt into ring slot kt & 3.  Lane p < 8 fetches the entry of
    // k-row 2 (p & 3) + (p >> 2), so that the four entries a half-wave needs (it loads the even or the
    // odd k-rows of the wave's chunks) lie side by side; the other lanes point outside the window and
    // store zeros.  Past the live rows the base is held at n: unused values.
    __device__ __forceinline__ void issue_index(int kt) const {
        const int lane = threadIdx.x & 63;
        const int base = min(kt * kBK2 + 8 * wl, n);
        const int voff = lane < 8 ? (base + 2 * (lane & 3) + (lane >> 2)) * 4 : kOutside;
        const uint32_t m0v = __builtin_amdgcn_readfirstlane(ring + 256u * (kt & 3));
        asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, 0 offen lds" ::"s"(m0v), "v"(voff), "s"(rsi)
                     : "memory");
    }
    __device__ __forceinline__ void chunk_load(int kt, uint32_t tile, int i, int row) const {
        const int lane = threadIdx.x & 63;
        const int k = kt * kBK2 + 8 * wl + 2 * i + (lane >> 5);
        const int voff = k < n ? row * ld_bytes + cvoff[i] : kOutside;
        lds_load16(rs, tile + 1024 * (4 * wl + i), voff);
    }
    // stages 0 and 1 of a tile: entries by scalar loads; the ring is started for stages 2 and 3
    __device__ __forceinline__ void issue_first(int kt, uint32_t tile) const {
        const int lane = threadIdx.x & 63;
        const int base = min(kt * kBK2 + 8 * wl, n);
        const int e0 = rows[base], e1 = rows[base + 1], e2 = rows[base + 2], e3 = rows[base + 3];
        const int e4 = rows[base + 4], e5 = rows[base + 5], e6 = rows[base + 6], e7 = rows[base + 7];
        issue_index(kt + 2);
        const bool odd = lane & 32;
        chunk_load(kt, tile, 0, odd ? e1 : e0);
        chunk_load(kt, tile, 1, odd ? e3 : e2);
        chunk_load(kt, tile, 2, odd ? e5 : e4);
        chunk_load(kt, tile, 3, odd ? e7 : e6);
    }
    // stage kt >= 2: its entries are in the ring (asked for at stage kt - 2, two stage barriers ago)
    __device__ __forceinline__ void issue(int kt, uint32_t tile) const {
        const int lane = threadIdx.x & 63;
        int4 v;
        // inline asm: the compiler knows of no store to the ring and would read it once, ahead of the loop
        asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                     : "=v"(v)
                     : "v"(ring + 256u * (kt & 3) + 16u * (lane >> 5))
                     : "memory");
        issue_index(kt + 2);
        chunk_load(kt, tile, 0, v.x);
        chunk_load(kt, tile, 1, v.y);
        chunk_load(kt, tile, 2, v.z);
        chunk_load(kt, tile, 3, v.w);
    }
    __device__ __forceinline__ bf16x8_t frag(const char *tile, int t, int s) const { return fr.read(tile, t, s); }
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

// 8 MFMAs with the next fragment reads threaded between them: one MFMA, two LDS reads, one
// MFMA, ...  The first MFMA goes out at once (right after a barrier the matrix pipe would
// otherwise idle while a wave issues its reads), and the reads ride in the shadow of the
// MFMAs.  Left alone the compiler sinks the reads below the MFMAs and every sub-step starts
// by waiting on LDS.
template <class POp, class QOp>
__device__ __forceinline__ void sub_step(Acc2 &acc, Frags &next, const Frags &cur, const POp &P, const QOp &Q,
                                         const char *stage, int s) {
    read_frags(next, P, Q, stage, s);
    mfma_block(acc, cur);
#pragma unroll
    for (int i = 0; i < kTP2 * kTQ2; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, kReadsPerMfma, 0);  // DS read
    }
    __builtin_amdgcn_sched_barrier(0);
}

// One resident stage (two 16-k sub-steps).  On entry `x` holds the last fragment set of the
// previous stage (zeros before the first): its MFMAs open this stage, so the matrix pipe has
// work while this stage's first fragment reads are in flight.  On exit `x` holds this
// stage's last fragment set, not yet multiplied.  The loads of the stage two ahead are
// issued between the two sub-steps (inline asm, stays where it is written).  At most two
// fragment sets are live next to the 128 accumulator registers.
template <class POp, class QOp>
__device__ __forceinline__ void stage_compute(Acc2 &acc, Frags &x, Frags &y, const POp &P, const QOp &Q,
                                              const char *stage, int kt_load, uint32_t stage_load, bool loader) {
    sub_step(acc, y, x, P, Q, stage, 0);
    if (loader) {
        P.issue(kt_load, stage_load);
        Q.issue(kt_load, stage_load + kOperandBytes);
    }
    __builtin_amdgcn_sched_barrier(0);
    sub_step(acc, x, y, P, Q, stage, 1);
}

// End of a stage.  Loaders wait until at most one stage's loads are outstanding (their share
// of the next stage has landed); everyone waits for its LDS reads; then the waves meet.  A
// bare s_barrier is used on purpose: __syncthreads() carries a fence for which the compiler
// drains every outstanding load, including the ones just issued two stages ahead.
template <int vm>   // vm: buffer loads per loader wave per stage (both operands)
__device__ __forceinline__ void stage_barrier(bool loader) {
    // s_waitcnt simm16: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]
    if (loader) __builtin_amdgcn_s_waitcnt((vm & 15) | (7 << 4) | (0 << 8) | ((vm >> 4) << 14));
    else __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));
    __builtin_amdgcn_s_barrier();
}

// stage 0 or 1 of a tile for either operand kind
template <class Op>
__device__ __forceinline__ void issue_first(const Op &op, int kt, uint32_t tile) {
    if constexpr (Op::kIndexed) op.issue_first(kt, tile);
    else op.issue(kt, tile);
}

// nk k-tiles of 32.  st0..st3: the four 32 KB LDS stages (distinct arrays).
// live_rows < 256: only output rows [0, live_rows) of the tile are needed (ragged tail of an
// expert's segment); the waves whose rows are all dead skip fragment reads and MFMAs and only
// keep their share of the loads and the barriers going.
template <class POp, class QOp>
__device__ __forceinline__ void mfma_mainloop2(Acc2 &acc, int nk, const POp &P, const QOp &Q, char *st0, char *st1,
                                               char *st2, char *st3, int live_rows = kTile) {
    if (nk <= 0) return;
    constexpr int NL = POp::kLoads + QOp::kLoads;
    const uint32_t a0 = lds_addr(st0), a1 = lds_addr(st1), a2 = lds_addr(st2), a3 = lds_addr(st3);
    const int wave_ = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // wave-uniform, and visibly so (scalar branch instead of exec masking)
    const bool loader = wave_ < kLoaderWaves;
    if ((wave_ / kWP2) * kWaveRowsQ >= live_rows) {
        // this wave's rows are not needed: keep the loads (if it is a loader) and the barriers going
        if (loader) {
            issue_first(P, 0, a0);
            issue_first(Q, 0, a0 + kOperandBytes);
            issue_first(P, 1, a1);
            issue_first(Q, 1, a1 + kOperandBytes);
        }
        stage_barrier<NL>(loader);
        for (int kt = 0; kt < nk; kt += 4) {
            if (loader) { P.issue(kt + 2, a2); Q.issue(kt + 2, a2 + kOperandBytes); }
            stage_barrier<NL>(loader);
            if (loader && kt + 1 < nk) { P.issue(kt + 3, a3); Q.issue(kt + 3, a3 + kOperandBytes); }
            stage_barrier<NL>(loader);
            if (loader && kt + 2 < nk) { P.issue(kt + 4, a0); Q.issue(kt + 4, a0 + kOperandBytes); }
            stage_barrier<NL>(loader);
            if (loader && kt + 3 < nk) { P.issue(kt + 5, a1); Q.issue(kt + 5, a1 + kOperandBytes); }
            stage_barrier<NL>(loader);
        }
        __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
        __builtin_amdgcn_s_barrier();
        return;
    }
    if (loader) {
        // stages 0 and 1 (a stage >= nk loads nothing useful but still counts)
        if constexpr (POp::kIndexed || QOp::kIndexed) {
            // an indexed operand's address arithmetic per stage is long: kept as a real loop, or the
            // compiler works out both stages ahead and spills the results
#pragma nounroll
            for (int st = 0; st < 2; ++st) {
                const uint32_t a = st == 0 ? a0 : a1;
                issue_first(P, st, a);
                issue_first(Q, st, a + kOperandBytes);
            }
        } else {
            issue_first(P, 0, a0);
            issue_first(Q, 0, a0 + kOperandBytes);
            issue_first(P, 1, a1);
            issue_first(Q, 1, a1 + kOperandBytes);
        }
    }
    stage_barrier<NL>(loader);
    Frags x, y;
#pragma unroll
    for (int i = 0; i < kTP2; ++i) x.a[i] = bf16x8_t{};
#pragma unroll
    for (int j = 0; j < kTQ2; ++j) x.b[j] = bf16x8_t{};
    // single loop exit (no break) keeps the accumulators in place
    for (int kt = 0; kt < nk; kt += 4) {
        stage_compute(acc, x, y, P, Q, st0, kt + 2, a2, loader);
        stage_barrier<NL>(loader);
        if (kt + 1 < nk) stage_compute(acc, x, y, P, Q, st1, kt + 3, a3, loader);
        stage_barrier<NL>(loader);
        if (kt + 2 < nk) stage_compute(acc, x, y, P, Q, st2, kt + 4, a0, loader);
        stage_barrier<NL>(loader);
        if (kt + 3 < nk) stage_compute(acc, x, y, P, Q, st3, kt + 5, a1, loader);
        stage_barrier<NL>(loader);
    }
    mfma_block(acc, x);
    // loads for stages past the end are still in flight: drain them, and meet, before anyone
    // reuses the stage buffers (the epilogues stage their stores through them)
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
    __builtin_amdgcn_s_barrier();
}

// ---------------------------------------------------------------------------
// Windowed form of the main loop: the reduction advances in windows of 64 k, held in two 64 KB
// buffers (P window 32 KB, Q window 32 KB).  Its reason is the K-contiguous operands: with 64 k
// per window a row of such an operand is 128 B, one whole cache line, and eight lanes of a tile
// load cover it with one request; with 32-k stages every line was asked for twice, half each
// time, one stage apart, and the kernels whose two operands are both of this kind ran into the
// request rate of the L2 (measured on the 16384-token layer: -16 % / -12 % on the two such
// kernels with whole-line requests and the same bytes).  The window after the current one is
// loaded while the current one is multiplied (measured: a shallower prefetch costs nothing),
// so every wait is "all my loads have landed" and nothing has to be counted.
// Transposed operands keep their 32-k tile form: a window is two such tiles back to back.
// ---------------------------------------------------------------------------
constexpr int kBK3 = 64;
constexpr int kWinBytes = kTile * kBK3 * 2;   // 32 KB: one operand's window
constexpr int kSuperBytes = 2 * kWinBytes;    // 64 KB: both operands
constexpr int kLoadsPerWindow = 16;           // tile loads per loader wave per window (8 per operand)

// K-contiguous 256-row window [256 rows][128 B]: 32 chunks of 1 KB (8 rows x 128 B), eight per
// loader wave; the 16-byte chunk c of row r sits at slot c ^ ((r >> 1) & 7) (KcFrag<64>'s
// conflict-free order), applied on the global side.  Chunk i of a wave is 32 rows below chunk
// i - 1 and has the same swizzle, so one per-lane offset and a stride describe all eight --
// unless the rows are gathered (ROWS = true): then each lane keeps the offsets of its eight rows.
// STASH (with ROWS): the eight row offsets live in LDS instead of registers (`stash`: 2 x 256 int4
// outside the tile buffers, one slot pair per loader thread) and are read back at every window issue;
// for kernels whose tile loop has no eight registers to spare.
// INSIDE (without ROWS): every row of the window exists (a weight panel), so the 32-row advance from
// chunk to chunk rides in the load's scalar offset and the lane keeps one offset register; otherwise
// (rows of an expert's segment, whose tail relies on the bounds check) each chunk has its own.
template <bool ROWS, bool STASH = false, bool INSIDE = false>
struct OpKC64 {
    static constexpr bool kIndexed = false, kWindowed = true;
    Src src[2];
    int wswitch;           // window from which src[1] takes over (two-phase reductions)
    int voff[(ROWS && !STASH) ? 8 : 1];
    int step;              // bytes between a lane's consecutive chunks (32 rows)
    int4 *stash;           // STASH: this thread's first slot; the second is 256 slots on
    KcFrag<kBK3> fr;
    int tid_;              // the thread index the lane constants were made from (see set_lane)
    __device__ __forceinline__ int lane_chunk() const {
        const int w = tid_ >> 6, lane = tid_ & 63;
        const int row0 = 8 * (w & 3) + (lane >> 3);
        return ((lane & 7) ^ ((row0 >> 1) & 7)) * 16;
    }
    __device__ __forceinline__ int lane_row(int i) const {   // row of this lane in its chunk i
        const int w = tid_ >> 6, lane = tid_ & 63;
        return 8 * (w & 3) + (lane >> 3) + 32 * i;
    }
    // The per-lane constants (load offset, fragment address parts, stash slot).  A kernel may call this
    // again for every tile with an opaque copy of threadIdx.x (opaque_tid()): the constants are then
    // made anew per tile and are not carried through the epilogue in registers.
    __device__ __forceinline__ void set_lane(int ld_bytes, int wave_base, int tid, int4 *stash_base = nullptr) {
        tid_ = tid;
        step = 32 * ld_bytes;
        if constexpr (!ROWS) voff[0] = lane_row(0) * ld_bytes + lane_chunk();   // (gathered rows: set_rows())
        stash = stash_base + (tid & 255);
        fr.init(wave_base, tid & 63);
    }
    __device__ __forceinline__ void init(int ld_bytes, int wave_base, int4 *stash_base = nullptr) {
        wswitch = 0x7fffffff;
        set_lane(ld_bytes, wave_base, threadIdx.x, stash_base);
    }
    // the byte offsets of this lane's eight gathered rows (ROWS)
    __device__ __forceinline__ void set_rows(const int (&v)[8]) {
        if constexpr (STASH) {
            if ((threadIdx.x >> 6) < kLoaderWaves) {
                stash[0] = make_int4(v[0], v[1], v[2], v[3]);
                stash[256] = make_int4(v[4], v[5], v[6], v[7]);
            }
        } else if constexpr (ROWS) {
#pragma unroll
            for (int i = 0; i < 8; ++i) voff[i] = v[i];
        }
    }
    // rows: only rows [0, rows) of the window are wanted (a multiple of 64; the rest is left as it is)
    __device__ __forceinline__ void issue_window(int J, uint32_t win, int rows = kTile) const {
        const bool second = J >= wswitch;
        const Src &s = second ? src[1] : src[0];
        const int Js = second ? J - wswitch : J;
        const int w = threadIdx.x >> 6;
        const rsrc_t r = src_rsrc(s, Js);
        if constexpr (!ROWS && INSIDE) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (rows == kTile || (i < 6 && 32 * i < rows))
                    lds_load16_soff(r, win + 1024 * ((w & 3) + kLoaderWaves * i), voff[0], i * step);
            return;
        }
        int vo[8];
        if constexpr (STASH) {
            // read as inline asm: left to the compiler, the two reads are hoisted out of the window loop
            // (nothing in it writes the stash) and the eight values are back in registers, or in scratch
            int4 a, b;
            asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:4096\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(a), "=&v"(b)
                         : "v"(lds_addr(stash))
                         : "memory");
            vo[0] = a.x; vo[1] = a.y; vo[2] = a.z; vo[3] = a.w;
            vo[4] = b.x; vo[5] = b.y; vo[6] = b.z; vo[7] = b.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) vo[i] = ROWS ? voff[(ROWS && !STASH) ? i : 0] : voff[0] + i * step;
        }
        if (rows == kTile) {   // the common case as straight-line code
#pragma unroll
            for (int i = 0; i < 8; ++i) lds_load16(r, win + 1024 * ((w & 3) + kLoaderWaves * i), vo[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 6; ++i)
                if (32 * i < rows)   // chunk i of a wave holds rows 32 i + 8 (w & 3) ..+7
                    lds_load16(r, win + 1024 * ((w & 3) + kLoaderWaves * i), vo[i]);
        }
    }
    __device__ __forceinline__ bf16x8_t frag_window(const char *win, int t, int u) const { return fr.read(win, t, u); }
};

// a 32-k tile operand as a window: tiles 2J and 2J+1 back to back
template <class Op>
__device__ __forceinline__ void win_issue(const Op &op, int J, uint32_t win, int rows = kTile) {
    if constexpr (Op::kWindowed) {
        op.issue_window(J, win, rows);
    } else {
        op.issue(2 * J, win);
        op.issue(2 * J + 1, win + kOperandBytes);
    }
}
template <class Op>
__device__ __forceinline__ bf16x8_t win_frag(const Op &op, const char *win, int t, int u) {
    if constexpr (Op::kWindowed) return op.frag_window(win, t, u);
    else return op.frag(win + (u >> 1) * kOperandBytes, t, u & 1);
}

template <class POp, class QOp>
__device__ __forceinline__ void sub_step3(Acc2 &acc, Frags &next, const Frags &cur, const POp &P, const QOp &Q,
                                          const char *pwin, const char *qwin, int u) {
#pragma unroll
    for (int i = 0; i < kTP2; ++i) next.a[i] = win_frag(P, pwin, i, u);
#pragma unroll
    for (int j = 0; j < kTQ2; ++j) next.b[j] = win_frag(Q, qwin, j, u);
    mfma_block(acc, cur);
#pragma unroll
    for (int i = 0; i < kTP2 * kTQ2; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, kReadsPerMfma, 0);  // DS read
    }
    __builtin_amdgcn_sched_barrier(0);
}

// End of a window: a loader's loads (the next window) have all landed, everyone's fragment reads
// are done, then the waves meet.  Bare s_barrier, as in stage_barrier().
__device__ __forceinline__ void window_barrier(bool loader) {
    if (loader) __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (0 << 8) | (0 << 14));
    else __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));
    __builtin_amdgcn_s_barrier();
}

// One resident window (four 16-k sub-steps).  `x` carries the last fragment set of the previous
// window in and this window's last one out, as in stage_compute(); the next window's loads go out
// into the buffer the previous window has just left, one operand before the first sub-step and
// the other after it (measured: all sixteen at once makes the loader waves late for the window's
// barrier; later than this shortens the time the loads have).
template <class POp, class QOp>
__device__ __forceinline__ void window_compute(Acc2 &acc, Frags &x, Frags &y, const POp &P, const QOp &Q,
                                               const char *pwin, const char *qwin, int Jnext, uint32_t pnext,
                                               uint32_t qnext, bool load_next, int qrows) {
    if (load_next) win_issue(P, Jnext, pnext);
    __builtin_amdgcn_sched_barrier(0);
    sub_step3(acc, y, x, P, Q, pwin, qwin, 0);
    if (load_next) win_issue(Q, Jnext, qnext, qrows);
    __builtin_amdgcn_sched_barrier(0);
    sub_step3(acc, x, y, P, Q, pwin, qwin, 1);
    sub_step3(acc, y, x, P, Q, pwin, qwin, 2);
    sub_step3(acc, x, y, P, Q, pwin, qwin, 3);
}

// nw windows of 64 k.  `lds`: the work-group's 128 KB.  The two P windows sit at 0 and 32 KB, the two
// Q windows at 64 and 96 KB: a window and its twin are 32 KB apart, which fits the 16-bit offset
// field of an LDS read, so one address register per operand and sub-step serves both buffers (with
// P and Q of a buffer side by side the twin was 64 KB away and had registers of its own: eight
// more, in kernels that have none to spare).  live_rows as in mfma_mainloop2().  Every wave passes
// the same barriers whatever its role: one after the first window's loads and one per window.
template <class POp, class QOp>
__device__ __forceinline__ void mfma_mainloop3(Acc2 &acc, int nw, const POp &P, const QOp &Q, char *lds,
                                               int live_rows = kTile) {
    if (nw <= 0) return;
    char *const pA = lds, *const pB = lds + kWinBytes, *const qA = lds + 2 * kWinBytes, *const qB = lds + 3 * kWinBytes;
    const uint32_t apA = lds_addr(pA), apB = lds_addr(pB), aqA = lds_addr(qA), aqB = lds_addr(qB);
    const int wave_ = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool loader = wave_ < kLoaderWaves;
    // rows of the Q window that some wave reads: whole 64-row blocks (a tail tile's dead rows are
    // not fetched at all: their loads, though out of range, would still take their turn in the
    // vector memory path, and a tail tile is bound by that path and its latency)
    const int qrows = min(kTile, (live_rows + kWaveRowsQ - 1) / kWaveRowsQ * kWaveRowsQ);
    if (loader) {
        // windows 0 and 1 go out together; only window 0 is waited for: it is in when at most window
        // 1's loads are outstanding, 16 per loader wave for a full window; a tail tile issues fewer
        // for Q, so there only window 1's P share (8) may remain
        if constexpr (POp::kIndexed || QOp::kIndexed) {
            // an indexed operand's address arithmetic per tile load is long: kept as a real loop, or the
            // compiler works it all out ahead and spills the results (reloads that wait on the loads)
#pragma nounroll
            for (int w = 0; w < 2; ++w)
                if (w < nw) {
                    win_issue(P, w, w ? apB : apA);
                    win_issue(Q, w, w ? aqB : aqA, qrows);
                }
        } else {
            win_issue(P, 0, apA);
            win_issue(Q, 0, aqA, qrows);
            if (nw > 1) {
                win_issue(P, 1, apB);
                win_issue(Q, 1, aqB, qrows);
            }
        }
        if (nw > 1 && qrows == kTile)
            __builtin_amdgcn_s_waitcnt((kLoadsPerWindow & 15) | (7 << 4) | (0 << 8) | ((kLoadsPerWindow >> 4) << 14));
        else if (nw > 1) __builtin_amdgcn_s_waitcnt((kLoadsPerWindow / 2) | (7 << 4) | (0 << 8) | (0 << 14));
        else __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (0 << 8) | (0 << 14));
    }
    __builtin_amdgcn_s_barrier();
    if ((wave_ / kWP2) * kWaveRowsQ >= live_rows) {
        // this wave's rows are not needed: keep the loads (if it is a loader) and the barriers going
        for (int J = 0; J < nw; J += 2) {
            if (loader && J > 0 && J + 1 < nw) { win_issue(P, J + 1, apB); win_issue(Q, J + 1, aqB, qrows); }
            window_barrier(loader);
            if (J + 1 < nw) {
                if (loader && J + 2 < nw) { win_issue(P, J + 2, apA); win_issue(Q, J + 2, aqA, qrows); }
                window_barrier(loader);
            }
        }
        return;
    }
    Frags x, y;
#pragma unroll
    for (int i = 0; i < kTP2; ++i) x.a[i] = bf16x8_t{};
#pragma unroll
    for (int j = 0; j < kTQ2; ++j) x.b[j] = bf16x8_t{};
    for (int J = 0; J < nw; J += 2) {
        window_compute(acc, x, y, P, Q, pA, qA, J + 1, apB, aqB, loader && J > 0 && J + 1 < nw, qrows);
        window_barrier(loader);
        if (J + 1 < nw) {
            window_compute(acc, x, y, P, Q, pB, qB, J + 2, apA, aqA, loader && J + 2 < nw, qrows);
            window_barrier(loader);
        }
    }
    mfma_block(acc, x);
}

// ---------------------------------------------------------------------------
// The same loop for a tail tile: at most 64 live rows (the last few rows of an expert's segment).
// Such a tile multiplies little and is bound by the latency of its weight windows, so the space the
// dead 192 rows of the Q windows would take holds a third window instead and the loads run two
// windows ahead.  `lds` is the work-group's whole 128 KB: P windows at 0, 32, 64 KB; Q windows (rows
// 0..63 only, 8 KB each) from 96 KB.  Only waves 0 and 1 hold live rows; waves 0-3 load.
// A loader wave issues kTailLoads per window, so "at most that many outstanding" is "the next
// window is in" as long as the one after it has been issued.
// ---------------------------------------------------------------------------
constexpr int kTailQBytes = kWaveRowsQ * kBK3 * 2;                       // 8 KB: 64 rows of a Q window
constexpr int kTailLoads = 8 + 8 * kWaveRowsQ / kTile;                   // 8 for P + 2 for Q
constexpr int kTailQBase = 3 * kWinBytes;

__device__ __forceinline__ void tail_barrier(bool loader, bool one_ahead) {
    if (!loader) __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));
    else if (one_ahead) __builtin_amdgcn_s_waitcnt((kTailLoads & 15) | (7 << 4) | (0 << 8) | ((kTailLoads >> 4) << 14));
    else __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (0 << 8) | (0 << 14));
    __builtin_amdgcn_s_barrier();
}

template <class POp, class QOp>
__device__ __forceinline__ void mfma_tail_loop3(Acc2 &acc, int nw, const POp &P, const QOp &Q, char *lds) {
    if (nw <= 0) return;
    const uint32_t a0 = lds_addr(lds);
    const int wave_ = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool loader = wave_ < kLoaderWaves;
    const bool live = wave_ / kWP2 == 0;
    auto issue = [&](int J, int slot) {
        win_issue(P, J, a0 + slot * kWinBytes);
        win_issue(Q, J, a0 + kTailQBase + slot * kTailQBytes, kWaveRowsQ);
    };
    if (loader) {
        if constexpr (POp::kIndexed || QOp::kIndexed) {
#pragma nounroll
            for (int w = 0; w < 2; ++w)
                if (w < nw) issue(w, w);
        } else {
            issue(0, 0);
            if (nw > 1) issue(1, 1);
        }
    }
    tail_barrier(loader, nw > 1);
    Frags x, y;
#pragma unroll
    for (int i = 0; i < kTP2; ++i) x.a[i] = bf16x8_t{};
#pragma unroll
    for (int j = 0; j < kTQ2; ++j) x.b[j] = bf16x8_t{};
    // window J sits in slot J % 3; window J + 2 goes into the slot window J - 1 has just left
    auto window = [&](int J, int slot) {
        const int nslot = slot == 0 ? 2 : slot - 1;   // (slot + 2) % 3
        if (loader && J + 2 < nw) issue(J + 2, nslot);
        __builtin_amdgcn_sched_barrier(0);
        if (live) {
            const char *pw = lds + slot * kWinBytes, *qw = lds + kTailQBase + slot * kTailQBytes;
            sub_step3(acc, y, x, P, Q, pw, qw, 0);
            sub_step3(acc, x, y, P, Q, pw, qw, 1);
            sub_step3(acc, y, x, P, Q, pw, qw, 2);
            sub_step3(acc, x, y, P, Q, pw, qw, 3);
        }
        tail_barrier(loader, J + 2 < nw);
    };
    for (int J = 0; J < nw; J += 3) {
        window(J, 0);
        if (J + 1 < nw) window(J + 1, 1);
        if (J + 2 < nw) window(J + 2, 2);
    }
    if (live) mfma_block(acc, x);
}

// Persistent work-groups.  A launch has one work-group per compute unit; each walks the tile
// list instead of ending after one tile, so a tile's stores drain while the next tile's first
// loads are in flight and no work-group launch sits between two tiles.  The XCD-aware order
// of xcd_tile_id() is kept: XCD x owns tile ids [x*per, (x+1)*per).  The first two tiles of a
// work-group are fixed by its index; later ones come from a per-XCD counter (zeroed before
// the launch), so that slow and fast compute units even out, or, where all tiles take about
// the same time, simply follow round-robin.  The queue runs two tiles ahead:
// while tile i is worked on, tile i+1 is already known (its coordinates are fetched a whole
// tile before they are needed), and tile i+2 is asked for between tile i's loop (all its loads
// drained) and its epilogue (whose duration hides most of the round trip of the vector atomic,
// and where the fragment registers are free to hold the answer).  (Pulling the next tile's
// first stages into L2 during the epilogue, with loads into an LDS sink, was measured: no gain.)
// `mailbox` is two ints of LDS outside the stage buffers (alternating, so that a wave that is
// still reading one tile's slot cannot see the next one's).
constexpr int kQueueThread = 0;

// DYNAMIC = false: plain round-robin (slot, slot + stride, ...), for kernels whose tiles all
// take about the same time; nothing is fetched, so no wave waits for an atomic's round trip.
template <bool DYNAMIC>
struct TileLoopT {
    int total, per, xcd, stride, iter, nxt;
    int *ctr;
    __device__ __forceinline__ TileLoopT(int total_, int *ctr_row)
        : total(total_), per((total_ + 7) >> 3), xcd(blockIdx.x & 7), stride(gridDim.x >> 3), iter(0), nxt(0),
          ctr(ctr_row + (blockIdx.x & 7)) {}
    __device__ __forceinline__ int first() const { return blockIdx.x >> 3; }
    __device__ __forceinline__ int second() const { return (blockIdx.x >> 3) + stride; }
    __device__ __forceinline__ bool valid(int slot) const { return slot < per && xcd * per + slot < total; }
    __device__ __forceinline__ int id(int slot) const { return xcd * per + slot; }
    // ask for the slot two after the current one; call after the tile loop
    __device__ __forceinline__ void prefetch() {
        if constexpr (DYNAMIC)
            if (threadIdx.x == kQueueThread) nxt = 2 * stride + atomicAdd(ctr, 1);
    }
    // end of a tile: every wave's LDS traffic of the epilogue is complete and the waves have
    // met before anyone loads the next tile into the stage buffers; returns the slot two after
    // the current one
    __device__ __forceinline__ int finish(volatile int *mailbox) {
        if constexpr (DYNAMIC) {
            volatile int *box = mailbox + (iter & 1);
            if (threadIdx.x == kQueueThread) *box = nxt;
            // not __syncthreads(): its fence would also wait for this tile's global stores
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            ++iter;
            return __builtin_amdgcn_readfirstlane(*box);   // wave-uniform, and visibly so: tile coordinates stay scalar
        } else {
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            ++iter;
            return first() + (iter + 1) * stride;
        }
    }
};
typedef TileLoopT<true> TileLoop;          // tiles of uneven length (weight gradients)

// The row-tiled kernels' loop: XCD x owns the share [share[x], share[x + 1]) of the row-tile list, times the
// column tiles (tiles that share an operand panel sit next to each other and so meet in one L2).  A
// work-group's first two tiles are fixed (its index and its index plus the stride), the rest come from
// the share's counter, asked for a tile ahead (prefetch() after the tile loop, finish() hands the answer
// to all waves through `mailbox`, two ints of LDS outside the stage buffers).  Results do not depend on
// who ran which tile.  Measured on the 16384-token layer against a fixed round-robin: -1.5 % (down
// projection) and -2 % (dXp), the others unchanged.  Listing the short tail tiles last in every share, so
// that they fill up the last round (13.5 tiles per compute unit: by tile counts alone worth 5-7 % on the
// SwiGLU and dH kernels), made every row-tiled kernel 1-8 % slower instead: a tail tile then meets its
// expert's weight panels cold, long after the full tiles that shared them.
// Two ways of cutting the L2's re-fetches of operand panels were measured there as well and
// dropped: short tiles last under a fixed round-robin (fetched bytes -7 % (SwiGLU) to -15 % (dXp), time
// +1-3 %), and making the work-groups of an XCD start each round of tiles together (a bounded wait on a
// per-XCD counter: fetched bytes -20 %, time +12-23 %).  An XCD's round of 32 tiles does not line up with
// an expert's 24-30 tiles, so even in lockstep most weight panels are fetched in two rounds, and the
// fabric was not what the kernels were waiting for.
struct RowTileLoop {
    int start, cnt, stride, iter, nxt;
    int *ctr;
    // share: 9 ints (row-tile units); npt: column tiles per row tile; ctr_row: the launch's 8 counters
    __device__ __forceinline__ RowTileLoop(const int32_t *share, int npt, int *ctr_row)
        : stride(gridDim.x >> 3), iter(0), nxt(0) {
        const int xcd = blockIdx.x & 7;
        start = share[xcd] * npt;
        cnt = (share[xcd + 1] - share[xcd]) * npt;
        ctr = ctr_row + xcd;
    }
    __device__ __forceinline__ int first() const { return blockIdx.x >> 3; }
    __device__ __forceinline__ int second() const { return (blockIdx.x >> 3) + stride; }
    __device__ __forceinline__ bool valid(int slot) const { return slot < cnt; }
    __device__ __forceinline__ int id(int slot) const { return start + slot; }
    // ask for the slot two after the current one; call after the tile loop
    __device__ __forceinline__ void prefetch() {
        if (threadIdx.x == kQueueThread) nxt = 2 * stride + atomicAdd(ctr, 1);
    }
    // end of a tile: every wave's LDS traffic of the epilogue is complete and the waves have met
    // before anyone loads the next tile into the stage buffers; returns the slot two after the
    // current one.  (Not __syncthreads(): its fence would also wait for this tile's global stores.)
    __device__ __forceinline__ int finish(volatile int *mailbox) {
        volatile int *box = mailbox + (iter & 1);
        if (threadIdx.x == kQueueThread) *box = nxt;
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        ++iter;
        return __builtin_amdgcn_readfirstlane(*box);   // wave-uniform, and visibly so: tile coordinates stay scalar
    }
};

// Epilogue staging.  The MFMA result layout gives a lane 4 consecutive features of ONE row
// per register quad, so direct stores are 16-byte pieces scattered over 32 rows per
// instruction and the vector memory path spends more time on them than the tile spent on
// arithmetic.  Instead a wave drops a 32-row block into its private LDS patch (the stage
// buffers are free by now) and stores it back out with consecutive lanes along a row:
// full 128/256-byte row segments per instruction.  The same patch serves to bring in
// row-contiguous loads (saved activations, old gradients) for per-quad use.
// ROWB = payload bytes per row (128 or 256); rows are padded by 16 B against bank conflicts.
// `tid` is the thread's index as the epilogue sees it: the kernels pass a copy of threadIdx.x that the
// compiler cannot trace back (opaque_tid()), so that the lane and row constants of the epilogue are
// worked out after the tile loop instead of being carried through it in registers the loop needs.
__device__ __forceinline__ int opaque_tid() {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

template <int ROWB>
struct RowStage {
    static constexpr int PITCH = ROWB + 16;
    static constexpr int LPR = ROWB / 16;   // lanes per row when moving rows
    static constexpr int RPI = 64 / LPR;    // rows per instruction
    static constexpr int BYTES = 32 * PITCH;
    char *base;
    int tid;
    __device__ __forceinline__ void put8(int q, int byte_off, uint2 v) const { *(uint2 *)(base + q * PITCH + byte_off) = v; }
    __device__ __forceinline__ void put16(int q, int byte_off, float4 v) const { *(float4 *)(base + q * PITCH + byte_off) = v; }
    __device__ __forceinline__ uint2 get8(int q, int byte_off) const { return *(const uint2 *)(base + q * PITCH + byte_off); }
    // rows [0, valid) of the patch -> out (byte pointer at row 0), row pitch ld_bytes
    __device__ __forceinline__ void flush(char *out, int64_t ld_bytes, int valid) const {
        const int lane = tid & 63, r = lane / LPR, c = lane % LPR;
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = i * RPI + r;
            const uint4 v = *(const uint4 *)(base + row * PITCH + c * 16);
            if (row < valid) {
                // non-temporal: the output is not read again by this kernel and should not displace
                // operand tiles in L2 (measured: 1-3 % on the row-tiled GEMMs, at the price of 3 % on
                // the much shorter kernels that read these rows next)
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), (u32x4 *)(out + row * ld_bytes + c * 16));
            }
        }
    }
    // same for f32 rows, adding what is already in memory (accumulate != 0)
    __device__ __forceinline__ void flush_f32(char *out, int64_t ld_bytes, int valid, int accumulate) const {
        const int lane = tid & 63, r = lane / LPR, c = lane % LPR;
#pragma unroll 2
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = i * RPI + r;
            float4 v = *(const float4 *)(base + row * PITCH + c * 16);
            if (row < valid) {
                float4 *dst = (float4 *)(out + row * ld_bytes + c * 16);
                if (accumulate) {
                    const float4 old = *dst;
                    v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
                }
                *dst = v;
            }
        }
    }
    // in (byte pointer at row 0) -> rows [0, valid) of the patch, in two halves so that a caller can
    // have the next block's rows in flight while it works on this one
    struct Rows {
        uint4 v[32 / RPI];
    };
    __device__ __forceinline__ Rows fetch(const char *in, int64_t ld_bytes, int valid) const {
        const int lane = tid & 63, r = lane / LPR, c = lane % LPR;
        Rows x;
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = i * RPI + r;
            x.v[i] = make_uint4(0u, 0u, 0u, 0u);
            if (row < valid) {
                // read once per launch: non-temporal, so the rows do not displace operand tiles in L2
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                x.v[i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4 *)(in + row * ld_bytes + c * 16)));
            }
        }
        return x;
    }
    __device__ __forceinline__ void deposit(const Rows &x) const {
        const int lane = tid & 63, r = lane / LPR, c = lane % LPR;
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) *(uint4 *)(base + (i * RPI + r) * PITCH + c * 16) = x.v[i];
    }
    __device__ __forceinline__ void fill(const char *in, int64_t ld_bytes, int valid) const {
        deposit(fetch(in, ld_bytes, valid));
    }
};

// the wave's private share (128 KB / waves) of the (now idle) stage buffers
__device__ __forceinline__ char *wave_patch(char *s0, char *s1, char *s2, char *s3, int tid) {
    const int w = tid >> 6;
    if constexpr (kWaves2 == 8) {
        char *b = (w >> 1) == 0 ? s0 : (w >> 1) == 1 ? s1 : (w >> 1) == 2 ? s2 : s3;
        return b + (w & 1) * 16384;
    } else {
        return w == 0 ? s0 : w == 1 ? s1 : w == 2 ? s2 : s3;
    }
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
                f(tp, tq, g, wp * 128 + tp * 32 + g * 8 + (lane >> 5) * 4, wq * kWaveRowsQ + tq * 32 + (lane & 31));
}

__device__ __forceinline__ uint64_t clamp_bytes(int64_t b) { return b <= 0 ? 0u : (uint64_t)b; }

}  // namespace r3
