// Dense steps of the replayed MoE layer on bf16 MFMA (gfx950):
//   router logits  s = x W_r                       (Section 4.1, first equation)
//   grouped SwiGLU expert FFN, forward              (the E_i of the output equation)
//   its data gradients and weight gradients, and the router weight gradient.
// Every kernel is one instance of the tile loop in r3_mfma.h with its own
// operand addressing and epilogue.  Expert segments are ragged: a small kernel
// turns `offsets` into a list of (expert, first row) row tiles on the device, so
// nothing returns to the host between the permutation and the contractions.
#include <type_traits>

#include "r3_kernels.h"
#include "r3_mfma.h"
#include "r3_mfma2.h"
#include "r3_topk.h"

namespace r3 {

// ---------------------------------------------------------------------------
// Tile table, built by one block per pass:
//   tiles[0] = number of row tiles; tiles[1] = number of reduction segments (a multiple of 8);
//   tiles[2 .. 2+64) = the tile counters of up to eight persistent launches (8 XCDs each, zeroed here);
//   tiles[kTileSeg ..)  = reduction segments (expert, row0, row1, slot), longest first, dealt out evenly to
//     the 8 XCD shares of a tile list;
//   tiles[kTileHot ..)  = number of split experts, then (expert, first slot, slots) for each;
//   tiles[kTileX .. +9) = where each XCD's share of the row tiles starts (and where the last one ends);
//   tiles[kTileHdr ..)  = row tiles as (expert, row0) pairs, experts ascending, rows ascending (tiles
//     that share a weight panel are neighbours and meet in one L2); XCD x's share is the eighth
//     [tiles[kTileX + x], tiles[kTileX + x + 1]) of them, which its work-groups take from a counter.
// The weight-gradient kernels' tiles last as long as their expert has rows: taken longest first from a
// shared counter, a heavily loaded expert no longer starts late and finishes alone.  A segment is an
// expert's whole row range, or, when `split_rows` > 0, one of ceil(n / split_rows) equal parts of it
// (a multiple of 32 rows each): under a skewed load one expert's reduction can be longer than a compute
// unit's fair share of the whole launch, and no order of whole experts balances that.  Part 0 of an
// expert has slot -1 (its product goes to the gradient itself), part p > 0 has its own slot >= 0 in a
// scratch array of partial products, which a second launch adds to the gradient in slot order, so the
// result does not depend on which work-group ran what.  Segments that only pad the list to a multiple of
// 8 have slot -2 and are skipped.  At most kMaxSplitSlots slots are handed out (the caller's split_rows
// >= S / kMaxSplitSlots guarantees that this is never the binding limit).
// ---------------------------------------------------------------------------
constexpr int kRowTokensPad = 64;   // zeros after the row->token list
constexpr int kMaxSplitSlots = 32;
constexpr int kMaxSegs = kMaxE + kMaxSplitSlots + 8;
constexpr int kTileX = 2 + 64;               // 9 ints: first row tile of every XCD's share, and the end
constexpr int kTileSeg = kTileX + 16;
constexpr int kTileHot = kTileSeg + 4 * kMaxSegs;
constexpr int kTileHdr = kTileHot + 1 + 3 * kMaxSplitSlots + 3;
__device__ __forceinline__ int *tile_counters(const int32_t *tiles, int launch) {
    return const_cast<int *>(tiles) + 2 + 8 * launch;
}
// position of the item of rank `rank` among n (a multiple of 8) when the list is cut into 8 contiguous
// shares: dealt in serpentine order, so that every share holds an equal mix, heaviest first
__device__ __forceinline__ int dealt_position(int rank, int n) {
    const int j = rank >> 3, c = rank & 7;
    return ((j & 1) ? 7 - c : c) * (n >> 3) + j;
}
// rnk[i] = number of items that come before item i when the n items are sorted by descending key, ties
// by index.  A block of 1024 threads; an item's comparisons are shared out among 1024 / n' threads (n' = n
// rounded up to a power of two) and added up in LDS.  (One thread per item walking all n keys is a
// chain of n dependent LDS reads: 6 us at n = 128.)
template <class Key>
__device__ __forceinline__ void block_ranks(int n, Key key, int32_t *rnk) {
    for (int i = threadIdx.x; i < n; i += 1024) rnk[i] = 0;
    __syncthreads();
    if (n <= 1024) {
        int np2 = 1;
        while (np2 < n) np2 <<= 1;
        const int sub = 1024 / np2, i = threadIdx.x % np2, part = threadIdx.x / np2;
        const int per = (n + sub - 1) / sub, o0 = min(n, part * per), o1 = min(n, o0 + per);
        if (i < n) {
            const int k = key(i);
            int r = 0;
            for (int o = o0; o < o1; ++o) {
                const int m = key(o);
                r += (m > k) || (m == k && o < i);
            }
            if (r) atomicAdd(&rnk[i], r);
        }
    } else {
        for (int i = threadIdx.x; i < n; i += 1024) {
            const int k = key(i);
            int r = 0;
            for (int o = 0; o < n; ++o) {
                const int m = key(o);
                r += (m > k) || (m == k && o < i);
            }
            rnk[i] = r;
        }
    }
    __syncthreads();
}

__global__ void __launch_bounds__(1024)
build_row_tiles_kernel(int E, int BQ, const int32_t *__restrict__ offsets, int32_t *__restrict__ tiles,
                       int split_rows, int S, int K, const int32_t *__restrict__ perm,
                       const float *__restrict__ gates, int32_t *__restrict__ tok, float *__restrict__ grow) {
    // Work-groups past the first make the row -> token list (and the per-row gates) of the same pass: the
    // two jobs wait for the same inputs and are both too short to be worth a launch of their own.
    if (blockIdx.x > 0) {
        const int r = (blockIdx.x - 1) * 1024 + threadIdx.x;
        if (r < S) {
            const int slot = perm[r];
            tok[r] = slot / K;
            if (gates) grow[r] = gates[slot];
        } else if (r < S + kRowTokensPad) {
            tok[r] = 0;
        }
        return;
    }
    __shared__ int32_t start[kMaxE + 1];
    __shared__ int32_t off[kMaxE + 1];
    __shared__ int32_t seg0[kMaxE + 1];     // first segment of expert e
    __shared__ int32_t seglen[kMaxSegs];    // rows of every segment (-1: padding)
    __shared__ int32_t rnk[kMaxSegs];
    __shared__ int32_t nseg_s;
    // the offsets come in once, in parallel (read one by one by a single thread they cost a memory
    // round trip each, and this kernel sits between two others on every pass)
    for (int e = threadIdx.x; e <= E; e += blockDim.x) off[e] = offsets[e];
    __syncthreads();
    // Row tiles, parts and split experts per expert, then their running sums over the experts: every
    // thread takes kMaxE / 1024 neighbouring experts and the block scans the threads' totals.  (One
    // thread adding them up one after the other pays an LDS round trip per expert: 6 us for 128 experts,
    // in a kernel that sits between two others on every pass.)
    constexpr int PER = kMaxE / 1024;
    constexpr int NS = 3;                    // scanned: row tiles, parts, split experts
    __shared__ int32_t scan[NS][1024];
    int nt[PER], np[PER], tot[NS] = {0, 0, 0};
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int e = PER * threadIdx.x + i;
        const int n = e < E ? off[e + 1] - off[e] : 0;
        nt[i] = (n + BQ - 1) / BQ;
        np[i] = e < E ? (split_rows > 0 ? max(1, (n + split_rows - 1) / split_rows) : 1) : 0;
        tot[0] += nt[i];
        tot[1] += np[i];
        tot[2] += np[i] > 1;
    }
    for (int k = 0; k < NS; ++k) scan[k][threadIdx.x] = tot[k];
    __syncthreads();
    for (int dlt = 1; dlt < 1024; dlt <<= 1) {
        int v[NS];
        for (int k = 0; k < NS; ++k) v[k] = (int)threadIdx.x >= dlt ? scan[k][threadIdx.x - dlt] : 0;
        __syncthreads();
        for (int k = 0; k < NS; ++k) scan[k][threadIdx.x] += v[k];
        __syncthreads();
    }
    const int ntiles = scan[0][1023];
    // more parts than there are slots for (the caller's split_rows rules that out): no splitting at all
    const bool split = scan[1][1023] - E <= kMaxSplitSlots;
    {
        int run[NS];
        for (int k = 0; k < NS; ++k) run[k] = scan[k][threadIdx.x] - tot[k];   // exclusive
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int e = PER * threadIdx.x + i;
            if (e < E) {
                start[e] = run[0];
                seg0[e] = split ? run[1] : e;
                if (split && np[i] > 1) {   // slots are handed out in expert order: segments before e minus experts before e
                    tiles[kTileHot + 1 + 3 * run[2]] = e;
                    tiles[kTileHot + 2 + 3 * run[2]] = run[1] - e;
                    tiles[kTileHot + 3 + 3 * run[2]] = np[i] - 1;
                }
            }
            run[0] += nt[i];
            run[1] += np[i];
            run[2] += np[i] > 1;
        }
    }
    if (threadIdx.x == 1023) {
        const int segs = split ? scan[1][1023] : E;
        start[E] = ntiles;
        seg0[E] = segs;
        tiles[0] = ntiles;
        tiles[kTileHot] = split ? scan[2][1023] : 0;
        nseg_s = (segs + 7) & ~7;
        tiles[1] = nseg_s;
    }
    if (threadIdx.x < 64) tiles[2 + threadIdx.x] = 0;
    __syncthreads();
    if (threadIdx.x <= 8) tiles[kTileX + threadIdx.x] = (int)(((int64_t)ntiles * threadIdx.x) >> 3);
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const int n = start[e + 1] - start[e];
        for (int i = 0; i < n; ++i) {
            tiles[kTileHdr + 2 * (start[e] + i)] = e;
            tiles[kTileHdr + 1 + 2 * (start[e] + i)] = off[e] + i * BQ;
        }
    }
    if (split_rows < 0) return;   // (a pass with no weight gradients needs no segments)
    const int nseg = nseg_s;
    // part lengths: equal parts, a multiple of 32 rows, the last one takes what is left
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const int n = off[e + 1] - off[e], parts = seg0[e + 1] - seg0[e];
        const int len = parts > 1 ? ((n + parts - 1) / parts + 31) & ~31 : n;
        for (int p = 0; p < parts; ++p) seglen[seg0[e] + p] = max(0, min(len, n - p * len));
    }
    for (int i = seg0[E] + threadIdx.x; i < nseg; i += blockDim.x) seglen[i] = -1;
    __syncthreads();
    // rank every segment by length (ties by position) and write it where it is dealt to
    block_ranks(nseg, [&](int i) { return seglen[i]; }, rnk);
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const int n = off[e + 1] - off[e], parts = seg0[e + 1] - seg0[e];
        const int len = parts > 1 ? ((n + parts - 1) / parts + 31) & ~31 : n;
        const int slot = seg0[e] - e;   // slots were handed out in expert order (used if parts > 1)
        for (int p = 0; p < parts; ++p) {
            const int i = seg0[e] + p, m = seglen[i];
            int32_t *sg = tiles + kTileSeg + 4 * dealt_position(rnk[i], nseg);
            const int r0 = off[e] + min(p * len, n);
            sg[0] = e;
            sg[1] = r0;
            sg[2] = r0 + m;
            sg[3] = p == 0 ? -1 : slot + p - 1;
        }
    }
    for (int i = seg0[E] + threadIdx.x; i < nseg; i += blockDim.x) {
        int32_t *sg = tiles + kTileSeg + 4 * dealt_position(rnk[i], nseg);
        sg[0] = 0; sg[1] = 0; sg[2] = 0; sg[3] = -2;
    }
}

static inline int max_row_tiles(int64_t S, int E, int BQ) { return (int)(S / BQ) + E; }
static inline int grid_for(int64_t tiles) { return (int)((tiles + 7) / 8 * 8); }

// Grid of a persistent launch: one work-group per compute unit of the current device (a
// multiple of 8, so that every XCD gets the same number), fewer when there are fewer tiles.
static int device_cus() {
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
        cus[dev] = n / 8 * 8;
    }
    return cus[dev];
}
static int persistent_grid(int64_t max_tiles) {
    const int cus = device_cus();
    const int64_t g = (max_tiles + 7) / 8 * 8;
    return (int)(g < cus ? g : cus);
}

__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
    return make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d));
}
__device__ __forceinline__ void unpack4(uint2 v, float *f) {
    f[0] = __uint_as_float(v.x << 16);
    f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16);
    f[3] = __uint_as_float(v.y & 0xffff0000u);
}

// ---------------------------------------------------------------------------
// FFN, first contraction + SwiGLU:  A = Xp Wg, B = Xp Wu, H = silu(A) * B.
// The P operand is two 128-feature sub-tiles, one of W_gate and one of W_up, at
// the same features, so a wave holds both pre-activations of a (row, feature)
// pair in the same lane: MFMA tiles 0,1 are gate, tiles 2,3 the matching up.
// What is saved for the backward are not A and B but the two factors its SwiGLU
// step multiplies dh with: FA = B silu'(A) (dA = dh FA) and FB = silu(A)
// (dB = dh FB); the sigmoid is in registers here anyway, and the backward's
// epilogue is left with two multiplications per element.
// ---------------------------------------------------------------------------
template <bool GATHER>
__global__ void __launch_bounds__(kThreads2, kMinWavesPerSimd)
ffn1_kernel(int S, int d, int F, const bf16_t *__restrict__ Xp, const int32_t *__restrict__ perm, int K, int T,
            const int32_t *__restrict__ offsets, const int32_t *__restrict__ tiles, const bf16_t *__restrict__ Wg,
            const bf16_t *__restrict__ Wu, bf16_t *__restrict__ H, bf16_t *__restrict__ FA, bf16_t *__restrict__ FB,
            const float *__restrict__ grow) {
    __shared__ __attribute__((aligned(1024))) char lds[2 * kSuperBytes];   // one piece: a tail tile lays it out differently
    char *const bufA = lds, *const bufB = lds + kSuperBytes;
    char *const s0 = bufA, *const s1 = bufA + kStageBytes, *const s2 = bufB, *const s3 = bufB + kStageBytes;
    constexpr int BF = 128;  // features per tile
    const int npt = F / BF;
    OpTR128x2 P;
    P.init(F * 2, 0, 64 * ((threadIdx.x >> 6) % kWP2));
    OpKC64<GATHER> Q;
    Q.init(d * 2, kWaveRowsQ * ((threadIdx.x >> 6) / kWP2));
    __shared__ int mailbox[2];
    RowTileLoop tl(tiles + kTileX, npt, tile_counters(tiles, 0));
    struct Tile {
        int e, row0, row_end, f0;
    };
    auto decode = [&](int slot_) {
        const int id = tl.id(slot_);
        const int tile = id / npt, pt = id - tile * npt;
        Tile t;
        t.e = tiles[kTileHdr + 2 * tile];
        t.row0 = tiles[kTileHdr + 1 + 2 * tile];
        t.row_end = offsets[t.e + 1];
        t.f0 = pt * BF;
        return t;
    };
    auto aim = [&](const Tile &t) {   // point the operands at a tile
        const int64_t wb = ((int64_t)d * F - t.f0) * 2;
        P.src[0] = Src{(const char *)(Wg + (int64_t)t.e * d * F + t.f0), clamp_bytes(wb), (uint32_t)(kBK2 * F * 2)};
        P.src[1] = Src{(const char *)(Wu + (int64_t)t.e * d * F + t.f0), clamp_bytes(wb), (uint32_t)(kBK2 * F * 2)};
        if constexpr (GATHER) {
            // dispatch folded into the tile load: `Xp` is x [T,d]; each lane's eight rows of the tile
            // are read from their tokens' rows (rows past the end of the permutation repeat the last
            // one; they are never stored)
            Q.src[0] = Src{(const char *)Xp, clamp_bytes((int64_t)T * d * 2), kBK3 * 2};
            const int chunk = Q.lane_chunk();
            int v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = (perm[min(t.row0 + Q.lane_row(i), S - 1)] / K) * (d * 2) + chunk;
            Q.set_rows(v);
        } else {
            Q.src[0] = Src{(const char *)(Xp + (int64_t)t.row0 * d), clamp_bytes((int64_t)(S - t.row0) * d * 2), kBK3 * 2};
        }
        Q.src[1] = Q.src[0];
    };
    if (!tl.valid(tl.first())) return;
    Tile cur = decode(tl.first());
    aim(cur);
    for (int slot = tl.first(), next = tl.second(); tl.valid(slot);) {
    // the next tile's coordinates are fetched now (scalar loads), a whole tile before their use
    const bool more = tl.valid(next);
    const Tile nxt = more ? decode(next) : cur;
    const int e = cur.e, row0 = cur.row0, row_end = cur.row_end, f0 = cur.f0;

    Acc2 acc;
    zero_acc2(acc);
    if (row_end - row0 <= kWaveRowsQ) mfma_tail_loop3(acc, d / kBK3, P, Q, lds);
    else mfma_mainloop3(acc, d / kBK3, P, Q, lds, row_end - row0);
    tl.prefetch();
    if (more) aim(nxt);   // here, so that the row-index loads of a gathered tile hide behind the epilogue

    // per wave: 64 rows x 64 features of H (and FA, FB), 32 rows at a time through LDS
    // (three patches, so that one tensor's stores and the next one's deposits overlap)
    const int tid = opaque_tid();
    const int lane = tid & 63, wq = (tid >> 6) / kWP2, wp = (tid >> 6) % kWP2;
    char *patch = wave_patch(s0, s1, s2, s3, tid);
    const int q = lane & 31;
    const bool save = FA != nullptr;
#pragma unroll
    for (int tq = 0; tq < kTQ2; ++tq) {
        const int brow = row0 + wq * kWaveRowsQ + tq * 32;            // first row of this block
        const int valid = min(32, row_end - brow);             // may be <= 0
        const int64_t o = ((int64_t)brow * F + f0 + wp * 64) * 2;  // byte offset of the block
        RowStage<128> sh{patch, tid}, sa{patch + RowStage<128>::BYTES, tid}, sb{patch + 2 * RowStage<128>::BYTES, tid};
        // grow != NULL: H leaves as g H, g the gate of the row's slot (the down projection then yields
        // gated rows and the gradient of W_down finds its row operand ready); FA and FB are not scaled
        const float gq = grow ? (brow + q < row_end ? grow[brow + q] : 0.0f) : 1.0f;
#pragma unroll
        for (int tp = 0; tp < 2; ++tp)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float h[4], fa[4], fb[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a = acc[tp][tq][4 * g + i], b = acc[tp + 2][tq][4 * g + i];
                    const float sg = sigmoid_fast(a);
                    fb[i] = a * sg;                                  // silu(a)
                    h[i] = gq * (fb[i] * b);
                    fa[i] = b * fmaf(fb[i], 1.0f - sg, sg);          // b silu'(a), silu'(a) = sg (1 + a (1 - sg))
                }
                const int bo = (tp * 32 + g * 8 + (lane >> 5) * 4) * 2;
                sh.put8(q, bo, pack4(h[0], h[1], h[2], h[3]));
                if (save) {
                    sa.put8(q, bo, pack4(fa[0], fa[1], fa[2], fa[3]));
                    sb.put8(q, bo, pack4(fb[0], fb[1], fb[2], fb[3]));
                }
            }
        sh.flush((char *)H + o, (int64_t)F * 2, valid);
        if (save) {
            sa.flush((char *)FA + o, (int64_t)F * 2, valid);
            sb.flush((char *)FB + o, (int64_t)F * 2, valid);
        }
    }
    const int after = tl.finish(mailbox);
    slot = next;
    next = after;
    cur = nxt;
    }
}

// ---------------------------------------------------------------------------
// Row-ragged contraction with a plain or SwiGLU-backward epilogue:
//   out[row][p0+p] = sum_k Q[row][k] * Pmat[e](p, k)
// MODE 0: Yp = H Wd          P from Wd[e] [F,d]  (TR: k rows, features c), K = F
// MODE 1: u = dy Wd^T        P from Wd[e] [F,d]  (KC: feature rows f),      K = d
//         The Q rows are the upstream gradient's rows read through the row -> token list (row r is
//         dy[tok[r]]): the gated copy g*dy of every slot is never written.  Epilogue, with g the
//         row's gate, FA = B silu'(A) and FB = silu(A) saved by the forward:
//           dA = g u FA,  dB = g u FB,  Hg = g H  (the row operand of dW_down = Hg^T dy),
//           wpart[row][2 pt + wp] = g * sum over this wave's 128 features of u H
//         The parts of a row add up to g <dy, o> = g dg (o = H Wd: <dy, H Wd> = <dy Wd^T, H>), which is
//         all the masked-softmax backward needs, so the expert outputs are not read again either.
//         GATED: the forward already stored g H in place of H (one-call forward); the parts are then
//         sums of u (g H) and nothing is written for H.
// MODE 2: dXp = dA Wg^T + dB Wu^T   P from Wg[e], Wu[e] [d,F] (KC: rows c), K = 2F
//         (two-phase reduction: first F over (dA, Wg), then F over (dB, Wu))
// ---------------------------------------------------------------------------
template <int MODE, bool GATED = false>
__global__ void __launch_bounds__(kThreads2, kMinWavesPerSimd)
rowgemm_kernel(int S, int d, int F, const bf16_t *__restrict__ Q0, const bf16_t *__restrict__ Q1,
               const int32_t *__restrict__ offsets, const int32_t *__restrict__ tiles,
               const bf16_t *__restrict__ W0, const bf16_t *__restrict__ W1, const bf16_t *__restrict__ FA,
               const bf16_t *__restrict__ FB, bf16_t *__restrict__ out0, bf16_t *__restrict__ out1,
               const int32_t *__restrict__ tok, int T, const float *__restrict__ grow,
               const bf16_t *__restrict__ Hs, bf16_t *__restrict__ out2, float *__restrict__ wpart) {
    __shared__ __attribute__((aligned(1024))) char lds[2 * kSuperBytes];   // one piece: a tail tile lays it out differently
    char *const bufA = lds, *const bufB = lds + kSuperBytes;
    char *const s0 = bufA, *const s1 = bufA + kStageBytes, *const s2 = bufB, *const s3 = bufB + kStageBytes;
    const int NOUT = (MODE == 1) ? F : d;  // width of the output
    const int KQ = (MODE == 1) ? d : F;    // width of the Q source rows
    const int npt = NOUT / kTile;
    const int nw = (MODE == 0) ? F / kBK3 : (MODE == 1) ? d / kBK3 : 2 * (F / kBK3);   // windows of 64 k
    const int wp0 = (threadIdx.x >> 6) % kWP2, wq0 = (threadIdx.x >> 6) / kWP2;
    // operand forms: the weights are feature-contiguous (TR) for MODE 0, K-contiguous otherwise
    typedef typename std::conditional<MODE == 0, OpTR256, OpKC64<false, false, true>>::type POp;
    constexpr bool GATHER = MODE == 1;     // Q rows through the row -> token list
    __shared__ int4 qstash[GATHER ? 2 * 256 : 1];   // the gathered rows' offsets (no registers to spare for them)
    POp P;
#ifndef R3_DH_STASH
#define R3_DH_STASH 1
#endif
    OpKC64<GATHER, GATHER && R3_DH_STASH> Q;
    if constexpr (MODE == 0) {
        P.kswitch = 0x7fffffff;
        P.init(d * 2, 0, 128 * wp0);
    } else {
        P.init((MODE == 1 ? d : F) * 2, 128 * wp0);
        if constexpr (MODE == 2) P.wswitch = F / kBK3;
    }
    Q.init(KQ * 2, kWaveRowsQ * wq0, qstash);
    if constexpr (MODE == 2) Q.wswitch = F / kBK3;
    __shared__ int mailbox[2];
    RowTileLoop tl(tiles + kTileX, npt, tile_counters(tiles, MODE == 1 ? 0 : 1));
    struct Tile {
        int e, row0, row_end, p0;
    };
    auto decode = [&](int slot_) {
        const int id = tl.id(slot_);
        const int tile = id / npt, pt = id - tile * npt;
        Tile t;
        t.e = tiles[kTileHdr + 2 * tile];
        t.row0 = tiles[kTileHdr + 1 + 2 * tile];
        t.row_end = offsets[t.e + 1];
        t.p0 = pt * kTile;
        return t;
    };
    auto aim = [&](const Tile &t) {   // point the operands at a tile
        const bf16_t *w0 = W0 + (int64_t)t.e * d * F;
        if constexpr (GATHER) {
            // each lane's eight rows of the tile come from their tokens' rows of Q0 [T, KQ] (rows past the
            // end of the list read token 0: the list is padded with zeros; they are never stored)
            Q.src[0] = Src{(const char *)Q0, clamp_bytes((int64_t)T * KQ * 2), kBK3 * 2};
            const int chunk = Q.lane_chunk();
            int v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = tok[min(t.row0 + Q.lane_row(i), S)] * (KQ * 2) + chunk;
            Q.set_rows(v);
        } else {
            Q.src[0] = Src{(const char *)(Q0 + (int64_t)t.row0 * KQ), clamp_bytes((int64_t)(S - t.row0) * KQ * 2), kBK3 * 2};
        }
        Q.src[1] = Q.src[0];
        if constexpr (MODE == 2)
            Q.src[1] = Src{(const char *)(Q1 + (int64_t)t.row0 * KQ), clamp_bytes((int64_t)(S - t.row0) * KQ * 2), kBK3 * 2};
        if constexpr (MODE == 0) {
            P.src[0] = Src{(const char *)(w0 + t.p0), clamp_bytes(((int64_t)d * F - t.p0) * 2), (uint32_t)(kBK2 * d * 2)};
            P.src[1] = P.src[0];
        } else if constexpr (MODE == 1) {
            P.src[0] = Src{(const char *)(w0 + (int64_t)t.p0 * d), clamp_bytes((int64_t)(F - t.p0) * d * 2), kBK3 * 2};
            P.src[1] = P.src[0];
        } else {
            const bf16_t *w1 = W1 + (int64_t)t.e * d * F;
            P.src[0] = Src{(const char *)(w0 + (int64_t)t.p0 * F), clamp_bytes((int64_t)(d - t.p0) * F * 2), kBK3 * 2};
            P.src[1] = Src{(const char *)(w1 + (int64_t)t.p0 * F), clamp_bytes((int64_t)(d - t.p0) * F * 2), kBK3 * 2};
        }
    };
    if (!tl.valid(tl.first())) return;
    Tile cur = decode(tl.first());
    if constexpr (GATHER) aim(cur);
    for (int slot = tl.first(), next = tl.second(); tl.valid(slot);) {
    // the next tile's coordinates are fetched now (scalar loads), a whole tile before their use
    const bool more = tl.valid(next);
    const Tile nxt = more ? decode(next) : cur;
    const int row0 = cur.row0, row_end = cur.row_end, p0 = cur.p0;
    if constexpr (!GATHER) aim(cur);
    if constexpr (MODE == 1) {
        // the operands' lane constants are made anew for every tile, from a thread index the compiler
        // cannot trace: kept across tiles they are live through the epilogue, the fullest part of this
        // kernel, and are then spilled, with reloads in the tile loop that wait on the tile loads
        const int t0 = opaque_tid();
        P.set_lane(d * 2, 128 * ((t0 >> 6) % kWP2), t0);
        Q.set_lane(KQ * 2, kWaveRowsQ * ((t0 >> 6) / kWP2), t0, qstash);
    }

    Acc2 acc;
    zero_acc2(acc);
    if (row_end - row0 <= kWaveRowsQ) mfma_tail_loop3(acc, nw, P, Q, lds);
    else mfma_mainloop3(acc, nw, P, Q, lds, row_end - row0);
    tl.prefetch();
    if constexpr (GATHER)
        if (more) aim(nxt);   // here, so that the row-index loads of the next tile hide behind the epilogue

    // per wave: 64 rows x 128 features, 32 rows at a time through LDS
    const int tid = opaque_tid();
    const int lane = tid & 63, wq = (tid >> 6) / kWP2, wp = (tid >> 6) % kWP2;
    RowStage<256> st{wave_patch(s0, s1, s2, s3, tid), tid};
    const int q = lane & 31;
    if constexpr (MODE == 1) {
        // Four rounds of 32 rows x 64 features, each in three phases: FA -> dA, FB -> dB, H -> g H and the
        // row's dot product.  A phase's rows come in row-contiguously into a patch, each lane replaces
        // exactly the quads it read, and the patch goes out row-contiguously.  The rows of the phase
        // after next are asked for while this one is worked on: two 4 KB blocks in flight per wave (a
        // whole round ahead, three blocks, cost the tile loop its registers).  A lane's 16 + 16 products
        // u H of one 32-row block belong to one row (q).
        typedef RowStage<128> Patch;
        const Patch sa{st.base, tid}, sb{st.base + Patch::BYTES, tid}, sh{st.base + 2 * Patch::BYTES, tid};
        constexpr int NPH = 3 * 2 * kTQ2;   // (GATED: the H phases only read)
        auto where = [&](int ph, int &valid) -> int64_t {
            const int r = ph / 3;
            const int brow = row0 + wq * kWaveRowsQ + (r >> 1) * 32;
            valid = min(32, row_end - brow);
            return ((int64_t)brow * NOUT + p0 + wp * 128) * 2 + (r & 1) * 128;
        };
        auto ask = [&](int ph) -> Patch::Rows {
            int valid;
            const int64_t o = where(ph, valid);
            const char *src = ph % 3 == 0 ? (const char *)FA : ph % 3 == 1 ? (const char *)FB : (const char *)Hs;
            return sa.fetch(src + o, (int64_t)NOUT * 2, valid);
        };
#ifndef R3_DH_AHEAD
#define R3_DH_AHEAD 1
#endif
        constexpr int AH = R3_DH_AHEAD;   // phases the row fetches run ahead (1 or 2)
        Patch::Rows rr[2] = {ask(0), ask(AH == 2 ? 1 : 0)};
        float gq = 0.0f, wsum = 0.0f;
#pragma unroll
        for (int ph = 0; ph < NPH; ++ph) {
            const int r = ph / 3, which = ph % 3, tq = r >> 1, half = r & 1;
            const int brow = row0 + wq * kWaveRowsQ + tq * 32;
            const Patch &sp = which == 0 ? sa : which == 1 ? sb : sh;
            int valid;
            const int64_t oh = where(ph, valid);
            sp.deposit(rr[AH == 2 ? (ph & 1) : 0]);
            if (ph + AH < NPH) rr[AH == 2 ? (ph & 1) : 0] = ask(ph + AH);
            if (which == 0 && half == 0) {
                gq = brow + q < row_end ? grow[brow + q] : 0.0f;
                wsum = 0.0f;
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int tp = half * 2 + t;
                    const int bo = (t * 32 + g * 8 + (lane >> 5) * 4) * 2;
                    float v[4], o[4];
                    unpack4(sp.get8(q, bo), v);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float u = acc[tp][tq][4 * g + i];
                        if (which == 2) {
                            wsum = fmaf(u, v[i], wsum);
                            o[i] = gq * v[i];
                        } else {
                            o[i] = gq * u * v[i];
                        }
                    }
                    if (!(GATED && which == 2)) sp.put8(q, bo, pack4(o[0], o[1], o[2], o[3]));
                }
            bf16_t *dst = which == 0 ? out0 : which == 1 ? out1 : out2;
            if (!(GATED && which == 2)) sp.flush((char *)dst + oh, (int64_t)NOUT * 2, valid);
            if (which == 2 && half == 1) {
                // the two lanes that hold row q (k-groups 0 and 1 of the MFMA layout) add up
                const float w = (GATED ? 1.0f : gq) * (wsum + __shfl_xor(wsum, 32, 64));
                if (lane < 32 && brow + q < row_end)
                    wpart[(int64_t)(brow + q) * (2 * npt) + 2 * (p0 / kTile) + wp] = w;
            }
        }
    } else {
#pragma unroll
        for (int tq = 0; tq < kTQ2; ++tq) {
            const int brow = row0 + wq * kWaveRowsQ + tq * 32;
            const int valid = min(32, row_end - brow);
            const int64_t o = ((int64_t)brow * NOUT + p0 + wp * 128) * 2;
#pragma unroll
            for (int tp = 0; tp < kTP2; ++tp)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    st.put8(q, (tp * 32 + g * 8 + (lane >> 5) * 4) * 2,
                            pack4(acc[tp][tq][4 * g], acc[tp][tq][4 * g + 1], acc[tp][tq][4 * g + 2],
                                  acc[tp][tq][4 * g + 3]));
            st.flush((char *)out0 + o, (int64_t)NOUT * 2, valid);
        }
    }
    const int after = tl.finish(mailbox);
    slot = next;
    next = after;
    cur = nxt;
    }
}

// ---------------------------------------------------------------------------
// Weight gradients:  out[e][q][p] (+)= sum_{r in expert e} Qs[r][q] * Ps[r][p]
// Both operands are [row][feature] matrices, so both tiles are TR; the k loop
// runs over the expert's rows and the buffer bound zero-fills the tail.
// ---------------------------------------------------------------------------
// GATHER: Ps is the un-permuted matrix [nrows, NPd] and row r of the reduction is its row tok[r]
// (dW_down = Hg^T dy straight from the upstream gradient: no per-slot copy of dy is read).
template <bool GATHER>
__global__ void __launch_bounds__(kThreads2, kMinWavesPerSimd)
wgrad_kernel(int NQd, int NPd, const bf16_t *__restrict__ Qs, const bf16_t *__restrict__ Ps,
             const int32_t *__restrict__ tok, int nrows, const int32_t *__restrict__ tiles,
             float *__restrict__ out, float *__restrict__ part, int accumulate, int *ctr) {
    __shared__ __attribute__((aligned(1024))) char s0[kStageBytes];
    __shared__ __attribute__((aligned(1024))) char s1[kStageBytes];
    __shared__ __attribute__((aligned(1024))) char s2[kStageBytes];
    __shared__ __attribute__((aligned(1024))) char s3[kStageBytes];
    __shared__ int mailbox[2];
    __shared__ __attribute__((aligned(256))) char ring[GATHER ? kIndexRingBytes : 16];
    const int nqt = NQd / kTile, npt = NPd / kTile;
    const int wp0 = (threadIdx.x >> 6) % kWP2, wq0 = (threadIdx.x >> 6) / kWP2;
    // operands are set up once; a tile only moves their source windows (column offset included)
    typename std::conditional<GATHER, OpTR256G, OpTR256>::type P;
    OpTR256 Q;
    Q.kswitch = 0x7fffffff;
    if constexpr (GATHER) {
        P.init(NPd * 2, 128 * wp0, ring);
    } else {
        P.kswitch = 0x7fffffff;
        P.init(NPd * 2, 0, 128 * wp0);
    }
    Q.init(NQd * 2, 0, kWaveRowsQ * wq0);
    // tiles of one reduction segment (an expert's rows, or one part of them) are neighbours in the list
    TileLoop tl(tiles[1] * nqt * npt, ctr);
    for (int slot = tl.first(), next = tl.second(); tl.valid(slot);) {
    const int id = tl.id(slot);
    const int eo = id / (nqt * npt);
    const int rem = id - eo * nqt * npt;
    const int32_t *sg = tiles + kTileSeg + 4 * eo;
    const int e = sg[0], r0 = sg[1], r1 = sg[2], pslot = sg[3];
    const int qt = rem / npt, pt = rem - qt * npt;
    const int q0 = qt * kTile, p0 = pt * kTile;
    if (pslot != -2) {   // (a segment that only pads the list has no tile)
    if constexpr (GATHER) {
        P.aim(Ps, (uint64_t)nrows * NPd * 2, p0 * 2, tok + r0, r1 - r0);
    } else {
        P.src[0] = Src{(const char *)(Ps + (int64_t)r0 * NPd + p0), clamp_bytes(((int64_t)(r1 - r0) * NPd - p0) * 2),
                       (uint32_t)(kBK2 * NPd * 2)};
        P.src[1] = P.src[0];
    }
    Q.src[0] = Src{(const char *)(Qs + (int64_t)r0 * NQd + q0), clamp_bytes(((int64_t)(r1 - r0) * NQd - q0) * 2),
                   (uint32_t)(kBK2 * NQd * 2)};
    Q.src[1] = Q.src[0];

    Acc2 acc;
    zero_acc2(acc);
    mfma_mainloop2(acc, (r1 - r0 + kBK2 - 1) / kBK2, P, Q, s0, s1, s2, s3);
    tl.prefetch();

    // per wave: 64 rows (q) x 128 features (p) of f32, as 32-row x 64-feature blocks through LDS
    const int tid = opaque_tid();
    const int lane = tid & 63, wq = (tid >> 6) / kWP2, wp = (tid >> 6) % kWP2;
    RowStage<256> st{wave_patch(s0, s1, s2, s3, tid), tid};
    const int q = lane & 31;
    // part 0 of an expert's rows goes to the gradient, a later part to its own slot of partial products
    char *o = (char *)(pslot < 0 ? out + (int64_t)e * NQd * NPd : part + (int64_t)pslot * NQd * NPd);
    const int add = pslot < 0 ? accumulate : 0;
#pragma unroll
    for (int tq = 0; tq < kTQ2; ++tq)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int tp = half * 2 + t;
                    st.put16(q, (t * 32 + g * 8 + (lane >> 5) * 4) * 4,
                             make_float4(acc[tp][tq][4 * g], acc[tp][tq][4 * g + 1], acc[tp][tq][4 * g + 2],
                                         acc[tp][tq][4 * g + 3]));
                }
            const int64_t off = ((int64_t)(q0 + wq * kWaveRowsQ + tq * 32) * NPd + p0 + wp * 128 + half * 64) * 4;
            st.flush_f32(o + off, (int64_t)NPd * 4, 32, add);
        }
    } else {
        tl.prefetch();
    }
    const int after = tl.finish(mailbox);
    slot = next;
    next = after;
    }
}

// ---------------------------------------------------------------------------
// Two weight gradients with a common row operand in one pass:
//   out0[e][q][p] (+)= sum_r Qs[r][q] * P0[r][p],   out1[e][q][p] (+)= sum_r Qs[r][q] * P1[r][p]
// (dW_gate and dW_up: Qs = Xp, P0 = dA, P1 = dB).  The P tile is two 128-feature sub-tiles, one
// of P0 and one of P1 at the same features, as in the forward SwiGLU kernel, so the Xp tile is
// fetched once for both products.
// ---------------------------------------------------------------------------
// GATHER: Qs is the un-permuted matrix [nrows, NQd] and row r of the reduction is its row tok[r]
// (dW_gate, dW_up straight from x: no gathered copy of the tokens is read).
template <bool GATHER>
__global__ void __launch_bounds__(kThreads2, kMinWavesPerSimd)
wgrad_pair_kernel(int NQd, int NPd, const bf16_t *__restrict__ Qs, const int32_t *__restrict__ tok, int nrows,
                  const bf16_t *__restrict__ P0, const bf16_t *__restrict__ P1, const int32_t *__restrict__ tiles,
                  float *__restrict__ out0, float *__restrict__ out1, float *__restrict__ part0,
                  float *__restrict__ part1, int accumulate, int *ctr) {
    __shared__ __attribute__((aligned(1024))) char s0[kStageBytes];
    __shared__ __attribute__((aligned(1024))) char s1[kStageBytes];
    __shared__ __attribute__((aligned(1024))) char s2[kStageBytes];
    __shared__ __attribute__((aligned(1024))) char s3[kStageBytes];
    __shared__ int mailbox[2];
    __shared__ __attribute__((aligned(256))) char ring[GATHER ? kIndexRingBytes : 16];
    constexpr int BF = 128;  // features of P0 (and of P1) per tile
    const int nqt = NQd / kTile, npt = NPd / BF;
    const int wp0 = (threadIdx.x >> 6) % kWP2, wq0 = (threadIdx.x >> 6) / kWP2;
    OpTR128x2 P;
    P.init(NPd * 2, 0, 64 * wp0);
    typename std::conditional<GATHER, OpTR256G, OpTR256>::type Q;
    if constexpr (GATHER) {
        Q.init(NQd * 2, kWaveRowsQ * wq0, ring);
    } else {
        Q.kswitch = 0x7fffffff;
        Q.init(NQd * 2, 0, kWaveRowsQ * wq0);
    }
    // reduction segments as in wgrad_kernel: an expert's rows or one part of them
    TileLoop tl(tiles[1] * nqt * npt, ctr);
    for (int slot = tl.first(), next = tl.second(); tl.valid(slot);) {
    const int id = tl.id(slot);
    const int eo = id / (nqt * npt);
    const int rem = id - eo * nqt * npt;
    const int32_t *sg = tiles + kTileSeg + 4 * eo;
    const int e = sg[0], r0 = sg[1], r1 = sg[2], pslot = sg[3];
    const int qt = rem / npt, pt = rem - qt * npt;
    const int q0 = qt * kTile, p0 = pt * BF;
    if (pslot != -2) {
    const uint64_t pbytes = clamp_bytes(((int64_t)(r1 - r0) * NPd - p0) * 2);
    P.src[0] = Src{(const char *)(P0 + (int64_t)r0 * NPd + p0), pbytes, (uint32_t)(kBK2 * NPd * 2)};
    P.src[1] = Src{(const char *)(P1 + (int64_t)r0 * NPd + p0), pbytes, (uint32_t)(kBK2 * NPd * 2)};
    if constexpr (GATHER) {
        Q.aim(Qs, (uint64_t)nrows * NQd * 2, q0 * 2, tok + r0, r1 - r0);
    } else {
        Q.src[0] = Src{(const char *)(Qs + (int64_t)r0 * NQd + q0), clamp_bytes(((int64_t)(r1 - r0) * NQd - q0) * 2),
                       (uint32_t)(kBK2 * NQd * 2)};
        Q.src[1] = Q.src[0];
    }

    Acc2 acc;
    zero_acc2(acc);
    mfma_mainloop2(acc, (r1 - r0 + kBK2 - 1) / kBK2, P, Q, s0, s1, s2, s3);
    tl.prefetch();

    // per wave: 64 rows (q) x 64 features (p) of each product, 32-row blocks through LDS
    const int tid = opaque_tid();
    const int lane = tid & 63, wq = (tid >> 6) / kWP2, wp = (tid >> 6) % kWP2;
    RowStage<256> st{wave_patch(s0, s1, s2, s3, tid), tid};
    const int q = lane & 31;
#pragma unroll
    for (int tq = 0; tq < kTQ2; ++tq)
#pragma unroll
        for (int half = 0; half < 2; ++half) {   // MFMA tiles 0,1: first product; 2,3: second
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int tp = half * 2 + t;
                    st.put16(q, (t * 32 + g * 8 + (lane >> 5) * 4) * 4,
                             make_float4(acc[tp][tq][4 * g], acc[tp][tq][4 * g + 1], acc[tp][tq][4 * g + 2],
                                         acc[tp][tq][4 * g + 3]));
                }
            char *o = (char *)(pslot < 0 ? (half ? out1 : out0) + (int64_t)e * NQd * NPd
                                         : (half ? part1 : part0) + (int64_t)pslot * NQd * NPd);
            const int64_t off = ((int64_t)(q0 + wq * kWaveRowsQ + tq * 32) * NPd + p0 + wp * 64) * 4;
            st.flush_f32(o + off, (int64_t)NPd * 4, 32, pslot < 0 ? accumulate : 0);
        }
    } else {
        tl.prefetch();
    }
    const int after = tl.finish(mailbox);
    slot = next;
    next = after;
    }
}

// ---------------------------------------------------------------------------
// Router logits  s[t][e] = sum_c x[t][c] Wr[c][e] (+ bias[e]), f32 out.
// ---------------------------------------------------------------------------
template <class TL>
__global__ void __launch_bounds__(TL::NT)
logits_kernel(int T, int d, int E, const bf16_t *__restrict__ x, const bf16_t *__restrict__ Wr,
              const float *__restrict__ bias, float *__restrict__ logits) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int npt = E / TL::BP;
    const int nqt = (T + TL::BQ - 1) / TL::BQ;
    const int id = blockIdx.x;
    if (id >= nqt * npt) return;
    const int qt = id / npt, pt = id - qt * npt;
    const int t0 = qt * TL::BQ, p0 = pt * TL::BP;
    auto fp = [&](int kt, int k, int c) -> uint4 {
        return ld16(Wr + (int64_t)(kt * TL::BK + k) * E + p0 + c * 8);
    };
    auto fq = [&](int kt, int r, int c) -> uint4 {
        return ld16(x + (int64_t)min(t0 + r, T - 1) * d + kt * TL::BK + c * 8);
    };
    f32x16_t acc[TL::TP][TL::TQ];
    zero_acc<TL>(acc);
    mfma_mainloop<TL, true, false>(acc, d / TL::BK, fp, fq, lds);
    for_each_quad<TL>([&](int tp, int tq, int g, int p, int q) {
        const int t = t0 + q;
        if (t >= T) return;
        float4 v = make_float4(acc[tp][tq][4 * g], acc[tp][tq][4 * g + 1], acc[tp][tq][4 * g + 2],
                               acc[tp][tq][4 * g + 3]);
        if (bias) {
            const float4 b = *(const float4 *)(bias + p0 + p);
            v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w;
        }
        *(float4 *)(logits + (int64_t)t * E + p0 + p) = v;
    });
}

// ---------------------------------------------------------------------------
// Router logits and replay gate in one kernel (Section 4.1: first equation and the replay-gate
// equation), for E = 128 experts: a work-group owns BQ tokens and all experts, so a token's whole
// logits row is in the work-group's accumulators.  The tile (plus bias) goes to LDS as [BQ][E] f32
// and never to memory unless the caller asks for it (logits_out).  Then 8 lanes take a token:
//   gates: g_j = exp(s[id_j] - m) / sum_i exp(s[id_i] - m) over the recorded ids (m their maximum);
//   agreement (optional, K <= 8): the token's own top-K mask from the row (the record kernel's
//   selection) against the mask of the recorded ids: shared experts and "same set".
// A recorded id >= E is clamped and raises R3_DATA_IDX_RANGE; a non-finite logit among the recorded
// ones raises R3_DATA_NONFINITE.  The block adds its agreement counts once (integer atomics).
// ---------------------------------------------------------------------------
template <class TL, typename IdxT>
__global__ void __launch_bounds__(TL::NT, 2)   // two work-groups per compute unit: twice the bytes in flight
gate_fused_kernel(int T, int d, int K, const bf16_t *__restrict__ x, const bf16_t *__restrict__ Wr,
                  const float *__restrict__ bias, const IdxT *__restrict__ idx, int64_t stride,
                  float *__restrict__ gates, float *__restrict__ logits_out, unsigned long long *agree,
                  int32_t *status) {
    constexpr int E = TL::BP, PITCH = E + 4;   // floats per LDS row (the pad spreads rows over the banks)
    static_assert(E == 128, "one work-group holds all experts");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    __shared__ unsigned long long part[TL::NWAVES][2];
    const int t0 = blockIdx.x * TL::BQ;
    auto fp = [&](int kt, int k, int c) -> uint4 { return ld16(Wr + (int64_t)(kt * TL::BK + k) * E + c * 8); };
    auto fq = [&](int kt, int r, int c) -> uint4 {
        return ld16(x + (int64_t)min(t0 + r, T - 1) * d + kt * TL::BK + c * 8);
    };
    f32x16_t acc[TL::TP][TL::TQ];
    zero_acc<TL>(acc);
    mfma_mainloop_ahead2<TL, true, false>(acc, d / TL::BK, fp, fq, lds);   // ends with a barrier: the stages are free
    float *sl = (float *)lds;
    for_each_quad<TL>([&](int tp, int tq, int g, int p, int q) {
        float4 v = make_float4(acc[tp][tq][4 * g], acc[tp][tq][4 * g + 1], acc[tp][tq][4 * g + 2],
                               acc[tp][tq][4 * g + 3]);
        if (bias) {
            const float4 b = *(const float4 *)(bias + p);
            v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w;
        }
        *(float4 *)(sl + q * PITCH + p) = v;
    });
    __syncthreads();
    if (logits_out)   // whole rows, 16 bytes per lane
        for (int i = threadIdx.x; i < TL::BQ * (E / 4); i += TL::NT) {
            const int q = i / (E / 4), c = i % (E / 4);
            if (t0 + q < T) *(float4 *)(logits_out + (int64_t)(t0 + q) * E + 4 * c) = *(const float4 *)(sl + q * PITCH + 4 * c);
        }
    const int sub = threadIdx.x & 7;
    int bad = 0;
    unsigned long long equal = 0, common = 0;
    for (int q = threadIdx.x >> 3; q < TL::BQ; q += TL::NT / 8) {
        const int t = t0 + q;
        const bool live = t < T;
        const float *row = sl + q * PITCH;
        const IdxT *id = idx + (int64_t)(live ? t : 0) * stride;
        // gate: slots sub, sub + 8, ... of the token
        float m = -INFINITY;
        for (int j = sub; j < K; j += 8) {
            int e = (int)id[j];
            if (e >= E) { bad |= R3_DATA_IDX_RANGE; e = E - 1; }
            const float z = row[e];
            if (!(fabsf(z) <= 3.4028235e38f)) bad |= R3_DATA_NONFINITE;
            m = fmaxf(m, z);
        }
        m = fmaxf(m, __shfl_xor(m, 1, 8));
        m = fmaxf(m, __shfl_xor(m, 2, 8));
        m = fmaxf(m, __shfl_xor(m, 4, 8));
        float den = 0.0f;
        for (int j = sub; j < K; j += 8) den += expf(row[min((int)id[j], E - 1)] - m);
        den += __shfl_xor(den, 1, 8);
        den += __shfl_xor(den, 2, 8);
        den += __shfl_xor(den, 4, 8);
        const float inv = 1.0f / den;
        if (live)
            for (int j = sub; j < K; j += 8) gates[(int64_t)t * K + j] = expf(row[min((int)id[j], E - 1)] - m) * inv;
        if (agree) {   // K <= 8 (checked by the host)
            constexpr int NV = E / 32;
            uint32_t key[NV][4];
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const float4 v = *(const float4 *)(row + 32 * i + 4 * sub);
                bool nf;
                key[i][0] = order_key(v.x, nf);
                key[i][1] = order_key(v.y, nf);
                key[i][2] = order_key(v.z, nf);
                key[i][3] = order_key(v.w, nf);
            }
            uint32_t own[NV], rec[NV];
            topk_mask8<NV>(key, K, sub, own);
            const int e = sub < K ? min((int)id[sub], E - 1) : -1;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                uint32_t w = (e >> 5) == i ? 1u << (e & 31) : 0u;   // e = -1 matches no word
                w |= group8_exchange<0>(w);
                w |= group8_exchange<1>(w);
                w |= group8_exchange<2>(w);
                rec[i] = w;
            }
            int shared = 0;
#pragma unroll
            for (int i = 0; i < NV; ++i) shared += __popc(own[i] & rec[i]);
            if (live && sub == 0) {
                common += (unsigned long long)shared;
                equal += shared == K;
            }
        }
    }
    if (bad && status) atomicOr(status, bad);
    if (agree) {
        equal = wave_sum(equal);
        common = wave_sum(common);
        const int w = threadIdx.x / kWave;
        if (lane_id() == 0) {
            part[w][0] = equal;
            part[w][1] = common;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned long long a0 = 0, a1 = 0;
            for (int i = 0; i < TL::NWAVES; ++i) {
                a0 += part[i][0];
                a1 += part[i][1];
            }
            if (a1) atomicAdd(agree + 1, a1);
            if (a0) atomicAdd(agree, a0);
        }
    }
}

// ---------------------------------------------------------------------------
// Router weight gradient, split over tokens.  ds arrives as [T, 2E] bf16 with
// dz split into hi (columns 0..E) and lo (columns E..2E) halves:
//   part[s][c][e'] = sum_{t in split s} x[t][c] * ds[t][e'],   e' in [0, 2E)
// followed by a fixed-order sum over the splits and over (hi, lo).
// (E below is the width of ds, i.e. twice the number of experts.)
// A work-group takes 128 hidden columns and, with E = 128 experts, the whole width of ds, so x is
// read once; 16 splits of the tokens fill the chip with d / 128 tiles each and leave 16 partial
// matrices (with 128 x 128 tiles and a split per 512 tokens x was read twice and the partials, 67 MB
// at 16384 tokens, moved more bytes than x itself).
// ---------------------------------------------------------------------------
template <class TL>
__global__ void __launch_bounds__(TL::NT)
dwr_partial_kernel(int T, int d, int E, int rows_per_split, const bf16_t *__restrict__ x,
                   const bf16_t *__restrict__ ds, float *__restrict__ part) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int nqt = d / TL::BQ, npt = E / TL::BP;
    const int id = blockIdx.x;
    const int sp = id / (nqt * npt);
    const int rem = id - sp * nqt * npt;
    const int qt = rem / npt, pt = rem - qt * npt;
    const int r0 = sp * rows_per_split, r1 = min(T, r0 + rows_per_split);
    const int q0 = qt * TL::BQ, p0 = pt * TL::BP;
    auto fp = [&](int kt, int k, int c) -> uint4 {
        const int r = r0 + kt * TL::BK + k;
        return r < r1 ? ld16(ds + (int64_t)r * E + p0 + c * 8) : zero16();
    };
    auto fq = [&](int kt, int k, int c) -> uint4 {
        const int r = r0 + kt * TL::BK + k;
        return r < r1 ? ld16(x + (int64_t)r * d + q0 + c * 8) : zero16();
    };
    f32x16_t acc[TL::TP][TL::TQ];
    zero_acc<TL>(acc);
    // bound by the stream of x: two k-tiles in flight per work-group
    mfma_mainloop_ahead2<TL, true, true>(acc, (max(r1 - r0, 0) + TL::BK - 1) / TL::BK, fp, fq, lds);
    float *o = part + (int64_t)sp * d * E;
    for_each_quad<TL>([&](int tp, int tq, int g, int p, int q) {
        *(float4 *)(o + (int64_t)(q0 + q) * E + p0 + p) =
            make_float4(acc[tp][tq][4 * g], acc[tp][tq][4 * g + 1], acc[tp][tq][4 * g + 2],
                        acc[tp][tq][4 * g + 3]);
    });
}

// out[c][e] (+)= sum_s part[s][c][e] + part[s][c][E+e]
__global__ void __launch_bounds__(256)
split_reduce_kernel(int d, int E, int nsplit, const float *__restrict__ part, float *__restrict__ out,
                    int accumulate) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)d * E) return;
    const int c = (int)(i / E), e = (int)(i - (int64_t)c * E);
    float acc = accumulate ? out[i] : 0.0f;
    for (int s = 0; s < nsplit; ++s) {
        const float *row = part + ((int64_t)s * d + c) * 2 * E;
        acc += row[e] + row[E + e];
    }
    out[i] = acc;
}

// ---------------------------------------------------------------------------
// The partial products of split reductions into their gradients: for every split expert, in slot order
// (a fixed order: the sum does not depend on the launch shape).  n4 = float4s per expert matrix; a
// second gradient with slots of its own (out1, part1) is optional.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
wgrad_parts_kernel(int64_t n4, const int32_t *__restrict__ tiles, float *__restrict__ out0,
                   const float *__restrict__ part0, float *__restrict__ out1, const float *__restrict__ part1) {
    const int hot = tiles[kTileHot];
    for (int j = 0; j < hot; ++j) {
        const int e = tiles[kTileHot + 1 + 3 * j], s0 = tiles[kTileHot + 2 + 3 * j], ns = tiles[kTileHot + 3 + 3 * j];
        for (int which = 0; which < (out1 ? 2 : 1); ++which) {
            float4 *o = (float4 *)(which ? out1 : out0) + (int64_t)e * n4;
            const float4 *p = (const float4 *)(which ? part1 : part0) + (int64_t)s0 * n4;
            for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
                 i += (int64_t)gridDim.x * blockDim.x) {
                float4 a = o[i];
                for (int q = 0; q < ns; ++q) {
                    const float4 b = p[(int64_t)q * n4 + i];
                    a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
                }
                o[i] = a;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
typedef TileCfg<128, 64, 2, 2, 64> TLLogits;   // router: 128 experts x 64 tokens
typedef TileCfg<128, 128, 2, 2, 64> TLDwr;     // router (large batches): 128 experts x 128 tokens
typedef TileCfg<256, 128, 2, 2, 64> TLDwrW;    // router wgrad: 256 columns of ds (hi, lo) x 128 hidden

bool mfma_ffn_supported(int d, int F) { return d % 256 == 0 && F % 256 == 0 && d >= 256 && F >= 256; }
bool mfma_router_supported(int d, int E) { return E % 128 == 0 && d % 128 == 0; }  // 2E % 128 for ds

size_t mfma_tiles_bytes(int64_t S, int E) {
    return align_up((size_t)(kTileHdr + 2 * (size_t)max_row_tiles(S, E, kTile)) * sizeof(int32_t), 256);
}

template <class K>
static void allow_lds(K kernel, int bytes) {
    (void)hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

hipError_t mfma_build_tiles(int E, const int32_t *offsets, int32_t *tiles, int split_rows, hipStream_t s) {
    build_row_tiles_kernel<<<1, 1024, 0, s>>>(E, kTile, offsets, tiles, split_rows, 0, 1, nullptr, nullptr, nullptr,
                                              nullptr);
    return hipGetLastError();
}

hipError_t mfma_build_tiles_and_row_tokens(int E, const int32_t *offsets, int32_t *tiles, int split_rows, int S, int K,
                                           const int32_t *perm, const float *gates, int32_t *tok, float *grow,
                                           hipStream_t s) {
    build_row_tiles_kernel<<<1 + (S + kRowTokensPad + 1023) / 1024, 1024, 0, s>>>(E, kTile, offsets, tiles, split_rows,
                                                                                  S, K, perm, gates, tok, grow);
    return hipGetLastError();
}

hipError_t mfma_ffn_forward(int64_t S, int d, int E, int F, const void *Xp, const int32_t *perm, int K, int T,
                            const int32_t *offsets, const int32_t *tiles, const void *Wg, const void *Wu,
                            const void *Wd, void *Yp, void *H, void *FA, void *FB, const float *grow,
                            hipStream_t s) {
    const int mt = max_row_tiles(S, E, kTile);
    {
        ProfScope ps(PROF_FFN1, s);
        if (perm)
            ffn1_kernel<true><<<persistent_grid((int64_t)mt * (F / 128)), kThreads2, 0, s>>>(
                (int)S, d, F, (const bf16_t *)Xp, perm, K, T, offsets, tiles, (const bf16_t *)Wg, (const bf16_t *)Wu,
                (bf16_t *)H, (bf16_t *)FA, (bf16_t *)FB, grow);
        else
            ffn1_kernel<false><<<persistent_grid((int64_t)mt * (F / 128)), kThreads2, 0, s>>>(
                (int)S, d, F, (const bf16_t *)Xp, perm, K, T, offsets, tiles, (const bf16_t *)Wg, (const bf16_t *)Wu,
                (bf16_t *)H, (bf16_t *)FA, (bf16_t *)FB, grow);
    }
    ProfScope ps(PROF_FFN2, s);
    rowgemm_kernel<0><<<persistent_grid((int64_t)mt * (d / kTile)), kThreads2, 0, s>>>(
        (int)S, d, F, (const bf16_t *)H, nullptr, offsets, tiles, (const bf16_t *)Wd, nullptr, nullptr, nullptr,
        (bf16_t *)Yp, nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr);
    return hipGetLastError();
}

hipError_t mfma_ffn_dh(int64_t S, int d, int E, int F, const void *dy, const int32_t *tok, int T, const float *grow,
                       const int32_t *offsets, const int32_t *tiles, const void *Wd, const void *FA, const void *FB,
                       const void *H, void *dA, void *dB, void *Hg, float *wpart, hipStream_t s) {
    const int mt = max_row_tiles(S, E, kTile);
    ProfScope ps(PROF_DH, s);
    const int grid = persistent_grid((int64_t)mt * (F / kTile));
    if (Hg)
        rowgemm_kernel<1, false><<<grid, kThreads2, 0, s>>>(
            (int)S, d, F, (const bf16_t *)dy, nullptr, offsets, tiles, (const bf16_t *)Wd, nullptr,
            (const bf16_t *)FA, (const bf16_t *)FB, (bf16_t *)dA, (bf16_t *)dB, tok, T, grow, (const bf16_t *)H,
            (bf16_t *)Hg, wpart);
    else   // H already holds the gate-scaled rows
        rowgemm_kernel<1, true><<<grid, kThreads2, 0, s>>>(
            (int)S, d, F, (const bf16_t *)dy, nullptr, offsets, tiles, (const bf16_t *)Wd, nullptr,
            (const bf16_t *)FA, (const bf16_t *)FB, (bf16_t *)dA, (bf16_t *)dB, tok, T, grow, (const bf16_t *)H,
            nullptr, wpart);
    return hipGetLastError();
}

hipError_t mfma_ffn_dxp(int64_t S, int d, int E, int F, const void *dA, const void *dB, const int32_t *offsets,
                        const int32_t *tiles, const void *Wg, const void *Wu, void *dXp, hipStream_t s) {
    const int mt = max_row_tiles(S, E, kTile);
    ProfScope ps(PROF_DXP, s);
    rowgemm_kernel<2><<<persistent_grid((int64_t)mt * (d / kTile)), kThreads2, 0, s>>>(
        (int)S, d, F, (const bf16_t *)dA, (const bf16_t *)dB, offsets, tiles, (const bf16_t *)Wg,
        (const bf16_t *)Wu, nullptr, nullptr, (bf16_t *)dXp, nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr);
    return hipGetLastError();
}

// Rows per part of a split reduction for a launch whose segments have `tiles_per_seg` tiles each: a tile
// should not last longer than a third of a compute unit's fair share of the launch (0: never split).
// Never below S / kMaxSplitSlots, so that the slots always suffice.
int mfma_wgrad_split_rows(int64_t S, int tiles_per_seg, size_t part_bytes_available, size_t bytes_per_slot) {
    if (part_bytes_available < (size_t)kMaxSplitSlots * bytes_per_slot) return 0;
    const int cus = device_cus();
    int64_t r = S * tiles_per_seg / (3 * (int64_t)cus);
    r = std::max<int64_t>(r, (S + kMaxSplitSlots - 1) / kMaxSplitSlots);
    r = std::max<int64_t>(r, 2048);
    r = (r + 31) / 32 * 32;
    return r >= S ? 0 : (int)r;
}

hipError_t mfma_wgrad(int E, int NQd, int NPd, const void *Qs, const void *Ps, const int32_t *tok, int nrows,
                      const int32_t *tiles, int launch, float *out, float *part, int accumulate, hipStream_t s) {
    const int64_t ntiles = (int64_t)(E + kMaxSplitSlots + 8) * (NQd / kTile) * (NPd / kTile);
    ProfScope ps(PROF_WGRAD, s);
    if (tok)
        wgrad_kernel<true><<<persistent_grid(ntiles), kThreads2, 0, s>>>(
            NQd, NPd, (const bf16_t *)Qs, (const bf16_t *)Ps, tok, nrows, tiles, out, part, accumulate,
            const_cast<int *>(tiles) + 2 + 8 * launch);
    else
        wgrad_kernel<false><<<persistent_grid(ntiles), kThreads2, 0, s>>>(
            NQd, NPd, (const bf16_t *)Qs, (const bf16_t *)Ps, nullptr, 0, tiles, out, part, accumulate,
            const_cast<int *>(tiles) + 2 + 8 * launch);
    if (part) wgrad_parts_kernel<<<512, 256, 0, s>>>((int64_t)NQd * NPd / 4, tiles, out, part, nullptr, nullptr);
    return hipGetLastError();
}

hipError_t mfma_wgrad_pair(int E, int NQd, int NPd, const void *Qs, const int32_t *tok, int nrows, const void *P0,
                           const void *P1, const int32_t *tiles, int launch, float *out0, float *out1, float *part,
                           int accumulate, hipStream_t s) {
    const int64_t ntiles = (int64_t)(E + kMaxSplitSlots + 8) * (NQd / kTile) * (NPd / 128);
    const int64_t n = (int64_t)NQd * NPd;
    float *part1 = part ? part + (int64_t)kMaxSplitSlots * n : nullptr;   // the second product's slots
    ProfScope ps(PROF_WGRAD_PAIR, s);
    if (tok)
        wgrad_pair_kernel<true><<<persistent_grid(ntiles), kThreads2, 0, s>>>(
            NQd, NPd, (const bf16_t *)Qs, tok, nrows, (const bf16_t *)P0, (const bf16_t *)P1, tiles, out0, out1, part,
            part1, accumulate, const_cast<int *>(tiles) + 2 + 8 * launch);
    else
        wgrad_pair_kernel<false><<<persistent_grid(ntiles), kThreads2, 0, s>>>(
            NQd, NPd, (const bf16_t *)Qs, nullptr, 0, (const bf16_t *)P0, (const bf16_t *)P1, tiles, out0, out1, part,
            part1, accumulate, const_cast<int *>(tiles) + 2 + 8 * launch);
    if (part) wgrad_parts_kernel<<<512, 256, 0, s>>>(n / 4, tiles, out0, part, out1, part1);
    return hipGetLastError();
}

// tok[r] = perm[r] / K for r < S (the token whose row sits at position r of the expert-sorted order),
// followed by `pad` zeros, so that index fetches one past a segment's end stay inside the array;
// grow[r] = gates[perm[r]], the gate of that row's slot (gates may be NULL: grow is then not written)
__global__ void __launch_bounds__(256) row_tokens_kernel(int S, int K, int pad, const int32_t *__restrict__ perm,
                                                         const float *__restrict__ gates, int32_t *__restrict__ tok,
                                                         float *__restrict__ grow) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r < S) {
        const int slot = perm[r];
        tok[r] = slot / K;
        if (gates) grow[r] = gates[slot];
    } else if (r < S + pad) {
        tok[r] = 0;
    }
}

size_t mfma_row_tokens_bytes(int64_t S) { return (size_t)(S + kRowTokensPad) * sizeof(int32_t); }

hipError_t mfma_row_tokens(int S, int K, const int32_t *perm, const float *gates, int32_t *tok, float *grow,
                           hipStream_t s) {
    row_tokens_kernel<<<(S + kRowTokensPad + 255) / 256, 256, 0, s>>>(S, K, kRowTokensPad, perm, gates, tok, grow);
    return hipGetLastError();
}

hipError_t mfma_router_logits(int T, int d, int E, const void *x, const void *Wr, const float *bias,
                              float *logits, hipStream_t s) {
    typedef TLLogits TL;
    allow_lds(logits_kernel<TL>, TL::LDS_BYTES);
    const int tiles = ((T + TL::BQ - 1) / TL::BQ) * (E / TL::BP);
    ProfScope ps(PROF_LOGITS, s);
    logits_kernel<TL><<<tiles, TL::NT, TL::LDS_BYTES, s>>>(T, d, E, (const bf16_t *)x, (const bf16_t *)Wr, bias,
                                                         logits);
    return hipGetLastError();
}

bool mfma_gate_fused_supported(int d, int E, int K, bool want_agreement) {
    return E == 128 && d % 64 == 0 && (!want_agreement || K <= 8);
}

template <class TL, typename IdxT>
static void launch_gate_fused(int T, int d, int K, const void *x, const void *Wr, const float *bias, const void *idx,
                              int64_t stride, float *gates, float *logits_out, int64_t *agree, int32_t *status,
                              hipStream_t s) {
    constexpr int LDS = TL::LDS_BYTES > TL::BQ * (TL::BP + 4) * 4 ? TL::LDS_BYTES : TL::BQ * (TL::BP + 4) * 4;
    allow_lds(gate_fused_kernel<TL, IdxT>, LDS);
    gate_fused_kernel<TL, IdxT><<<(T + TL::BQ - 1) / TL::BQ, TL::NT, LDS, s>>>(
        T, d, K, (const bf16_t *)x, (const bf16_t *)Wr, bias, (const IdxT *)idx, stride, gates, logits_out,
        (unsigned long long *)agree, status);
}

hipError_t mfma_gate_fused(int T, int d, int E, int K, const void *x, const void *Wr, const float *bias,
                           const void *idx, int idx_dtype, int64_t stride, float *gates, float *logits_out,
                           int64_t *agree, int32_t *status, hipStream_t s) {
    ProfScope ps(PROF_GATE, s);
    // The kernel lives on bytes in flight (one token tile per work-group, k-tiles in sequence): 128-token
    // tiles keep 64 KB of x on its way per compute unit; below 32768 tokens they would leave compute
    // units without a tile, so there 64-token tiles
    const bool big = T >= 32768;
    if (idx_dtype == R3_IDX_U8) {
        if (big) launch_gate_fused<TLDwr, uint8_t>(T, d, K, x, Wr, bias, idx, stride, gates, logits_out, agree, status, s);
        else launch_gate_fused<TLLogits, uint8_t>(T, d, K, x, Wr, bias, idx, stride, gates, logits_out, agree, status, s);
    } else {
        if (big) launch_gate_fused<TLDwr, uint16_t>(T, d, K, x, Wr, bias, idx, stride, gates, logits_out, agree, status, s);
        else launch_gate_fused<TLLogits, uint16_t>(T, d, K, x, Wr, bias, idx, stride, gates, logits_out, agree, status, s);
    }
    return hipGetLastError();
}

static int dwr_splits(int T) {
    int s = (T + 511) / 512;
    return s < 1 ? 1 : (s > 16 ? 16 : s);
}
size_t mfma_dwr_ws_bytes(int T, int d, int E) {
    return align_up((size_t)dwr_splits(T) * d * 2 * E * sizeof(float), 256);
}

hipError_t mfma_dwr(int T, int d, int E, const void *x, const void *ds, float *part, float *dWr, int accumulate,
                    hipStream_t s) {
    const int ns = dwr_splits(T);
    typedef TLDwrW TL;
    int rows = (T + ns - 1) / ns;
    rows = (rows + TL::BK - 1) / TL::BK * TL::BK;
    allow_lds(dwr_partial_kernel<TL>, TL::LDS_BYTES);
    ProfScope ps(PROF_DWR, s);
    dwr_partial_kernel<TL><<<ns * (d / TL::BQ) * (2 * E / TL::BP), TL::NT, TL::LDS_BYTES, s>>>(
        T, d, 2 * E, rows, (const bf16_t *)x, (const bf16_t *)ds, part);
    const int64_t n = (int64_t)d * E;
    split_reduce_kernel<<<(int)((n + 255) / 256), 256, 0, s>>>(d, E, ns, part, dWr, accumulate);
    return hipGetLastError();
}

}  // namespace r3
