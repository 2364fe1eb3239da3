// Router-mask cache of Section 4.2 of arxiv 2510.11370: routing masks kept beside a paged KV cache.
// Pages hold P tokens, token-major (one token's L*K ids are contiguous, so a decode step appends one
// piece per sequence); a block table maps (sequence, position / P) to a page, and a prefix shared by
// several sequences is the same page ids in their tables.  Two HBM-bound copies:
//   append: new ids (any layer / token strides)  ->  page slots
//   gather: page slots of a packed batch of sequences  ->  one layer-major record [L][T][K],
//           transposed through LDS so that both the page reads and the record writes are contiguous.
// Data moves in units of U bytes (the largest power of two <= 16 that divides K ids and every stride).
#include <algorithm>
#include <initializer_list>

#include "r3_kernels.h"

namespace r3 {
namespace {

constexpr int kTokTile = 64;  // tokens per work-group of the gather

template <int U> struct UnitOf;
template <> struct UnitOf<1> { typedef uint8_t type; };
template <> struct UnitOf<2> { typedef uint16_t type; };
template <> struct UnitOf<4> { typedef uint32_t type; };
template <> struct UnitOf<8> { typedef uint2 type; };
template <> struct UnitOf<16> { typedef uint4 type; };

// first sequence s with start[s + 1] > t  (start ascending, start[nseq] = T > t)
__device__ __forceinline__ int sequence_of(const int32_t *start, int nseq, int t) {
    int lo = 0, hi = nseq - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (start[mid + 1] > t) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// row (in tokens) of (sequence, position) inside the page pool, or -1
__device__ __forceinline__ int64_t page_row(const int32_t *block_table, int nseq, int max_blocks, int P,
                                            int64_t num_pages, int seq, int pos) {
    if (seq < 0 || seq >= nseq || pos < 0 || pos / P >= max_blocks) return -1;
    const int page = block_table[(int64_t)seq * max_blocks + pos / P];
    if (page < 0 || page >= num_pages) return -1;
    return (int64_t)page * P + pos % P;
}

// One thread per (token, layer, unit of the router's ids), unit fastest: a token's page row is written
// as one contiguous run.
template <int U>
__global__ void __launch_bounds__(256)
cache_append_kernel(int64_t n, int L, int S, int P, char *pages, int64_t num_pages, const int32_t *block_table,
                    int nseq, int max_blocks, const int32_t *seq_id, const int32_t *position, const char *src,
                    int64_t layer_bytes, int64_t token_bytes, int32_t *status) {
    typedef typename UnitOf<U>::type unit_t;
    const int64_t per_token = (int64_t)L * S;
    const int64_t total = n * per_token;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < total; v += (int64_t)gridDim.x * 256) {
        const int64_t i = v / per_token;
        const int ls = (int)(v - i * per_token);
        const int l = ls / S, sub = ls - l * S;
        const int64_t row = page_row(block_table, nseq, max_blocks, P, num_pages, seq_id[i], position[i]);
        if (row < 0) {
            if (ls == 0 && status) atomicOr(status, R3_DATA_CACHE_ADDR);
            continue;
        }
        const unit_t u = *(const unit_t *)(src + l * layer_bytes + i * token_bytes + (int64_t)sub * U);
        *(unit_t *)(pages + (row * per_token + ls) * U) = u;
    }
}

// Layer-major sources (token stride below the layer stride, e.g. the [L][n][K] that per-layer recording
// leaves): the transposition runs through LDS like the gather's, in the other direction.  Work-group =
// kTokTile consecutive new tokens x a chunk of LC layers; phase 1 reads, per layer, the tile's tokens
// (consecutive threads, consecutive source addresses when the source is packed), phase 2 writes each
// token's LC*S units into its page row as one run.
template <int U>
__global__ void __launch_bounds__(256)
cache_append_tiled_kernel(int64_t n, int L, int S, int LC, int P, char *pages, int64_t num_pages,
                          const int32_t *block_table, int nseq, int max_blocks, const int32_t *seq_id,
                          const int32_t *position, const char *src, int64_t layer_bytes, int64_t token_bytes,
                          int32_t *status) {
    typedef typename UnitOf<U>::type unit_t;
    extern __shared__ __align__(16) char smem[];
    __shared__ int64_t row_of[kTokTile];
    unit_t *tile = (unit_t *)smem;
    const int64_t i0 = (int64_t)blockIdx.x * kTokTile;
    const int l0 = blockIdx.y * LC;
    const int nl = min(LC, L - l0);
    const int nt = (int)min((int64_t)kTokTile, n - i0);
    const int pitch = (LC * S) | 1;
    if (threadIdx.x < kTokTile) {
        int64_t row = -1;
        if ((int)threadIdx.x < nt) {
            row = page_row(block_table, nseq, max_blocks, P, num_pages, seq_id[i0 + threadIdx.x],
                           position[i0 + threadIdx.x]);
            if (row < 0 && blockIdx.y == 0 && status) atomicOr(status, R3_DATA_CACHE_ADDR);
        }
        row_of[threadIdx.x] = row;
    }
    const int span = nt * S;
    for (int v = threadIdx.x; v < nl * span; v += 256) {
        const int l = v / span, ts = v - l * span;
        const int tok = ts / S, sub = ts - tok * S;
        tile[tok * pitch + l * S + sub] =
            *(const unit_t *)(src + (l0 + l) * layer_bytes + (i0 + tok) * token_bytes + (int64_t)sub * U);
    }
    __syncthreads();
    const int run = nl * S;
    for (int v = threadIdx.x; v < nt * run; v += 256) {
        const int tok = v / run, c = v - tok * run;
        const int64_t row = row_of[tok];
        if (row >= 0) *(unit_t *)(pages + ((row * L + l0) * S + c) * U) = tile[tok * pitch + c];
    }
}

// Work-group = kTokTile tokens x a chunk of LC layers.  Phase 1 reads each token's LC*S units from its
// page row (consecutive threads, consecutive units); phase 2 writes, per layer, the kTokTile*S units of
// the tile's tokens (consecutive threads, consecutive addresses of the record).  LDS row pitch is odd
// in units, so the strided phase-2 reads spread over the banks.
template <int U>
__global__ void __launch_bounds__(256)
cache_gather_kernel(int T, int L, int S, int LC, int P, const char *pages, int64_t num_pages,
                    const int32_t *block_table, int nseq, int max_blocks, const int32_t *seq_start, char *out,
                    int32_t *status) {
    typedef typename UnitOf<U>::type unit_t;
    extern __shared__ __align__(16) char smem[];
    __shared__ int64_t row_of[kTokTile];
    unit_t *tile = (unit_t *)smem;
    const int t0 = blockIdx.x * kTokTile;
    const int l0 = blockIdx.y * LC;
    const int nl = min(LC, L - l0);
    const int nt = min(kTokTile, T - t0);
    const int pitch = (LC * S) | 1;
    if (threadIdx.x < kTokTile) {
        int64_t row = -1;
        if ((int)threadIdx.x < nt) {
            const int t = t0 + threadIdx.x;
            const int s = sequence_of(seq_start, nseq, t);
            row = page_row(block_table, nseq, max_blocks, P, num_pages, s, t - seq_start[s]);
            if (row < 0 && blockIdx.y == 0 && status) atomicOr(status, R3_DATA_CACHE_ADDR);
        }
        row_of[threadIdx.x] = row;
    }
    __syncthreads();
    const int run = nl * S;  // units of one token in this chunk
    for (int v = threadIdx.x; v < nt * run; v += 256) {
        const int tok = v / run, c = v - tok * run;
        const int64_t row = row_of[tok];
        unit_t u = {};
        if (row >= 0) u = *(const unit_t *)(pages + ((row * L + l0) * S + c) * U);
        tile[tok * pitch + c] = u;
    }
    __syncthreads();
    const int span = nt * S;  // units of one layer in this tile
    for (int v = threadIdx.x; v < nl * span; v += 256) {
        const int l = v / span, ts = v - l * span;
        const int tok = ts / S, sub = ts - tok * S;
        *(unit_t *)(out + (((int64_t)(l0 + l) * T + t0) * S + ts) * U) = tile[tok * pitch + l * S + sub];
    }
}

// layers per chunk: the LDS tile of kTokTile tokens stays within 48 KiB
int layers_per_chunk(int L, int S, int U) {
    const int lc = (int)std::min<int64_t>(L, (48 * 1024 / (kTokTile * U) - 1) / S);
    return lc < 1 ? 1 : lc;
}

int pick_unit(int64_t router_bytes, std::initializer_list<int64_t> others) {
    int u = 16;
    while (u > 1) {
        bool ok = router_bytes % u == 0;
        for (int64_t o : others) ok = ok && (o % u == 0);
        if (ok) break;
        u >>= 1;
    }
    return u;
}

}  // namespace

hipError_t launch_cache_append(int idx_bytes, int L, int K, int P, void *pages, int64_t num_pages,
                               const int32_t *block_table, int nseq, int max_blocks, int64_t n,
                               const int32_t *seq_id, const int32_t *position, const void *idx_new,
                               int64_t layer_stride, int64_t token_stride, int32_t *status, hipStream_t s) {
    if (n == 0) return hipSuccess;
    const int64_t rb = (int64_t)K * idx_bytes;
    const int U = pick_unit(rb, {layer_stride * idx_bytes, token_stride * idx_bytes, (int64_t)(uintptr_t)pages,
                                 (int64_t)(uintptr_t)idx_new});
    const int S = (int)(rb / U);
    ProfScope ps(PROF_CACHE_APPEND, s);
    if (token_stride < layer_stride && L > 1) {
        const int LC = layers_per_chunk(L, S, U);
        const size_t lds = (size_t)kTokTile * ((LC * S) | 1) * U;
        dim3 grid((unsigned)((n + kTokTile - 1) / kTokTile), (L + LC - 1) / LC);
#define R3_APPEND_T(UU)                                                                                        \
    cache_append_tiled_kernel<UU><<<grid, 256, lds, s>>>(n, L, S, LC, P, (char *)pages, num_pages, block_table, \
                                                         nseq, max_blocks, seq_id, position,                   \
                                                         (const char *)idx_new, layer_stride * idx_bytes,      \
                                                         token_stride * idx_bytes, status)
        switch (U) {
            case 16: R3_APPEND_T(16); break;
            case 8: R3_APPEND_T(8); break;
            case 4: R3_APPEND_T(4); break;
            case 2: R3_APPEND_T(2); break;
            default: R3_APPEND_T(1); break;
        }
#undef R3_APPEND_T
        return hipGetLastError();
    }
    const int64_t total = n * L * S;
    const int grid = (int)std::min<int64_t>((total + 255) / 256, 1 << 16);
#define R3_APPEND(UU)                                                                                          \
    cache_append_kernel<UU><<<grid, 256, 0, s>>>(n, L, S, P, (char *)pages, num_pages, block_table, nseq,      \
                                                 max_blocks, seq_id, position, (const char *)idx_new,          \
                                                 layer_stride * idx_bytes, token_stride * idx_bytes, status)
    switch (U) {
        case 16: R3_APPEND(16); break;
        case 8: R3_APPEND(8); break;
        case 4: R3_APPEND(4); break;
        case 2: R3_APPEND(2); break;
        default: R3_APPEND(1); break;
    }
#undef R3_APPEND
    return hipGetLastError();
}

hipError_t launch_cache_gather(int idx_bytes, int L, int K, int P, const void *pages, int64_t num_pages,
                               const int32_t *block_table, int nseq, int max_blocks, const int32_t *seq_start,
                               int T, void *out, int32_t *status, hipStream_t s) {
    if (T == 0) return hipSuccess;
    const int64_t rb = (int64_t)K * idx_bytes;
    const int U = pick_unit(rb, {(int64_t)(uintptr_t)pages, (int64_t)(uintptr_t)out});
    const int S = (int)(rb / U);
    const int LC = layers_per_chunk(L, S, U);
    const size_t lds = (size_t)kTokTile * ((LC * S) | 1) * U;
    dim3 grid((T + kTokTile - 1) / kTokTile, (L + LC - 1) / LC);
    ProfScope ps(PROF_CACHE_GATHER, s);
#define R3_GATHER(UU)                                                                                          \
    cache_gather_kernel<UU><<<grid, 256, lds, s>>>(T, L, S, LC, P, (const char *)pages, num_pages, block_table, \
                                                   nseq, max_blocks, seq_start, (char *)out, status)
    switch (U) {
        case 16: R3_GATHER(16); break;
        case 8: R3_GATHER(8); break;
        case 4: R3_GATHER(4); break;
        case 2: R3_GATHER(2); break;
        default: R3_GATHER(1); break;
    }
#undef R3_GATHER
    return hipGetLastError();
}

}  // namespace r3
