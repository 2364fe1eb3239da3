// Per-kernel timing with HIP events and the calibration kernels (measurement aids, see
// include/r3_profile.h).
#include <atomic>
#include <mutex>
#include <vector>

#include "r3_kernels.h"
#include "r3_profile.h"

namespace r3 {
namespace {
constexpr int kPool = 512;
struct TagState {
    std::vector<hipEvent_t> start, stop;
    int used = 0;
};
std::mutex g_mu;
std::atomic<bool> g_on{false};   // read without the lock by every launch: off means "touch nothing"
TagState g_tags[PROF_NTAGS];
const char *kNames[PROF_NTAGS] = {"record_topk", "router_logits", "replay_gate", "permute_index",
                                  "gather_rows", "ffn1_swiglu", "ffn2_down", "combine", "gate_backward",
                                  "router_wgrad", "ffn_dh", "ffn_wgrad_down", "ffn_dxp", "dx_finish",
                                  "ffn_wgrad_gate_up", "routing_diff", "policy_discrepancy",
                                  "mask_cache_append", "mask_cache_gather", "agreement"};
}  // namespace

ProfScope::ProfScope(int tag_, hipStream_t s_) : tag(tag_), slot(-1), s(s_) {
    if (!g_on.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_on.load(std::memory_order_relaxed)) return;
    TagState &t = g_tags[tag];
    if (t.used >= kPool) return;
    if ((int)t.start.size() <= t.used) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
        t.start.push_back(a);
        t.stop.push_back(b);
    }
    slot = t.used++;
    (void)hipEventRecord(t.start[slot], s);
}

ProfScope::~ProfScope() {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lk(g_mu);
    (void)hipEventRecord(g_tags[tag].stop[slot], s);
}

// 16 bytes per thread per iteration, grid-stride: the reference point for traffic counters
__global__ void __launch_bounds__(256) calib_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src,
                                                         size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

typedef __bf16 cal_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float cal_f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned short cal_u16x8_t __attribute__((ext_vector_type(8)));

// the accumulator/fragment shape of the expert GEMMs' inner step, fed from registers only
__global__ void __launch_bounds__(512, 2) calib_mfma_kernel(int iters, int rnd, float *sink) {
    cal_bf16x8_t a[4], b[2];
    uint32_t h = (threadIdx.x + blockIdx.x * 977u) * 2654435761u;
    for (int i = 0; i < 6; ++i) {
        cal_u16x8_t u;
        for (int j = 0; j < 8; ++j) {
            h = h * 1664525u + 1013904223u;
            // finite bf16 values of either sign with varied mantissas, or the constant 1.0
            u[j] = rnd ? (unsigned short)(0x3c00u + ((h >> 9) & 0x83ffu)) : (unsigned short)0x3f80u;
        }
        if (i < 4) a[i] = __builtin_bit_cast(cal_bf16x8_t, u);
        else b[i - 4] = __builtin_bit_cast(cal_bf16x8_t, u);
    }
    cal_f32x16_t acc[4][2];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.0f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    if (s == 1.2345678f) *sink = s;  // keeps the loop alive
}

// The expert GEMMs' instruction mix without their synchronisation: per 8 MFMAs a wave reads 6 fragments
// (ds_read_b128) from LDS, and per two such steps the work-group brings 32 KB into LDS with direct
// global->LDS loads from a 1 MiB (cache-resident) source.  No barriers, no epilogue, no HBM misses: the rate
// a perfect schedule of the same mix would reach under the machine's power limit.  LDS holds varied bf16
// bit patterns; the loads race with the reads on purpose (only the traffic matters, every value is finite).
__global__ void __launch_bounds__(512, 2) calib_mix_kernel(int iters, const uint32_t *src, float *sink) {
    __shared__ __attribute__((aligned(16))) char lds[4][32768];
    uint32_t h = (threadIdx.x + blockIdx.x * 977u) * 2654435761u;
    for (int i = threadIdx.x; i < 4 * 32768 / 4; i += 512) {
        h = h * 1664525u + 1013904223u;
        ((uint32_t *)lds)[i] = (0x3c00u + ((h >> 9) & 0x83ffu)) | ((0x3c00u + ((h >> 3) & 0x83ffu)) << 16);
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    cal_f32x16_t acc[4][2];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    cal_bf16x8_t a[4], b[2];
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)src, (short)0, 1 << 20, 0x00020000);
    for (int it = 0; it < iters; ++it) {
        const char *st = lds[it & 3] + (w & 1) * 8192;
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = *(const cal_bf16x8_t *)(st + i * 1024 + lane * 16);
#pragma unroll
        for (int i = 0; i < 2; ++i) b[i] = *(const cal_bf16x8_t *)(st + 16384 + i * 1024 + lane * 16);
        if (it & 1) {
            char *dst = lds[(it + 2) & 3];
#pragma unroll
            for (int c = 0; c < 4; ++c)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    r, (__attribute__((address_space(3))) void *)(dst + c * 8192 + w * 1024), 16,
                    ((it * 4 + c) * 8192 + (int)threadIdx.x * 16) & ((1 << 20) - 1), 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0);
    float s = 0.0f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    if (s == 1.2345678f) *sink = s;
}

// The same for the other tile shape the GEMM header can be built for: 4 waves of 128 x 128 per work-group
// (one per SIMD, 256 accumulator registers each).  Per 16 MFMAs a wave reads 8 fragments -- a third fewer LDS
// bytes per FLOP -- and the work-group's global->LDS traffic per FLOP is the same (per 32 MFMAs of each wave it
// brings 32 KB).  Same FLOP per iteration and work-group as calib_mix_kernel (4 waves x 16 MFMAs).
__global__ void __launch_bounds__(256) calib_mix4_kernel(int iters, const uint32_t *src, float *sink) {
    __shared__ __attribute__((aligned(16))) char lds[4][32768];
    uint32_t h = (threadIdx.x + blockIdx.x * 977u) * 2654435761u;
    for (int i = threadIdx.x; i < 4 * 32768 / 4; i += 256) {
        h = h * 1664525u + 1013904223u;
        ((uint32_t *)lds)[i] = (0x3c00u + ((h >> 9) & 0x83ffu)) | ((0x3c00u + ((h >> 3) & 0x83ffu)) << 16);
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    cal_f32x16_t acc[4][4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    cal_bf16x8_t a[4], b[4];
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)src, (short)0, 1 << 20, 0x00020000);
    for (int it = 0; it < iters; ++it) {
        const char *st = lds[it & 3];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = *(const cal_bf16x8_t *)(st + (w & 1) * 4096 + i * 1024 + lane * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) b[i] = *(const cal_bf16x8_t *)(st + 16384 + (w >> 1) * 4096 + i * 1024 + lane * 16);
        if (it & 1) {
            char *dst = lds[(it + 2) & 3];
#pragma unroll
            for (int c = 0; c < 8; ++c)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    r, (__attribute__((address_space(3))) void *)(dst + c * 4096 + w * 1024), 16,
                    ((it * 8 + c) * 4096 + (int)threadIdx.x * 16) & ((1 << 20) - 1), 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0);
    float s = 0.0f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    if (s == 1.2345678f) *sink = s;
}

static int calib_grid() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) dev = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    return n;
}
}  // namespace r3

using namespace r3;

extern "C" {

int r3_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (on)
        for (auto &t : g_tags) t.used = 0;
    g_on.store(on != 0, std::memory_order_relaxed);
    return R3_OK;
}

int r3_profile_tags(void) { return PROF_NTAGS; }

const char *r3_profile_name(int tag) { return (tag >= 0 && tag < PROF_NTAGS) ? kNames[tag] : ""; }

int r3_profile_read(int tag, double *total_ms, int *launches) {
    if (tag < 0 || tag >= PROF_NTAGS || !total_ms || !launches) return R3_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    TagState &t = g_tags[tag];
    double sum = 0.0;
    for (int i = 0; i < t.used; ++i) {
        if (hipEventSynchronize(t.stop[i]) != hipSuccess) return R3_ERR_HIP;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, t.start[i], t.stop[i]) != hipSuccess) return R3_ERR_HIP;
        sum += ms;
    }
    *total_ms = sum;
    *launches = t.used;
    return R3_OK;
}

int r3_profile_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return R3_ERR_INVALID_ARG;
    if (bytes == 0) return R3_OK;
    size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    calib_copy_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>((uint4 *)dst, (const uint4 *)src, n);
    return hipGetLastError() == hipSuccess ? R3_OK : R3_ERR_HIP;
}

int r3_profile_mfma(int iters, int random_operands, float *sink, void *stream) {
    if (iters < 1 || iters > (1 << 24) || !sink) return R3_ERR_INVALID_ARG;
    calib_mfma_kernel<<<dim3(calib_grid()), dim3(512), 0, (hipStream_t)stream>>>(iters, random_operands, sink);
    return hipGetLastError() == hipSuccess ? R3_OK : R3_ERR_HIP;
}

int r3_profile_gemm_mix(int shape, int iters, const void *src_1mib, float *sink, void *stream) {
    if (iters < 1 || iters > (1 << 24) || !sink || !src_1mib || ((uintptr_t)src_1mib & 15) || shape < 0 || shape > 1)
        return R3_ERR_INVALID_ARG;
    if (shape == 1)
        calib_mix4_kernel<<<dim3(calib_grid()), dim3(256), 0, (hipStream_t)stream>>>(iters, (const uint32_t *)src_1mib,
                                                                                   sink);
    else
        calib_mix_kernel<<<dim3(calib_grid()), dim3(512), 0, (hipStream_t)stream>>>(iters, (const uint32_t *)src_1mib, sink);
    return hipGetLastError() == hipSuccess ? R3_OK : R3_ERR_HIP;
}

double r3_profile_mfma_flops(int iters) {
    return 2.0 * 32 * 32 * 16 * 8.0 * (double)iters * 8.0 * (double)calib_grid();
}
}
