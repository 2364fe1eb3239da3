// Shared device helpers for the gfx950 kernels of the replayed MoE layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "r3.h"

namespace r3 {

constexpr int kWave = 64;
constexpr int kMaxE = 4096;
constexpr int kMaxK = 64;

typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// f32 -> bf16, round to nearest even (NaN stays NaN): the gfx950 conversion instruction
// (v_cvt_pk_bf16_f32), which the compiler selects for this vector conversion.  The integer
// sequence it replaces cost about a dozen VALU operations per pair and dominated the GEMM
// epilogues.
typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float hw_f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const hw_f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, hw_bf16x2_t));
}

__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.0f) & 0xffffu); }

// element load/store by activation dtype
template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

__device__ __forceinline__ float sigmoidf_(float a) { return 1.0f / (1.0f + expf(-a)); }

// sigmoid from the hardware exp2 and reciprocal (about 2 ulp): for results that are rounded
// to bf16 right away.  exp(-a) = exp2(-a * log2(e)).
__device__ __forceinline__ float sigmoid_fast(float a) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(a * -1.44269504088896f));
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
template <typename T> __device__ __forceinline__ T wave_max(T v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        T w = __shfl_xor(v, o, kWave);
        v = w > v ? w : v;
    }
    return v;
}

// read one recorded expert id
template <typename IdxT>
__device__ __forceinline__ int load_idx(const void *idx, int64_t stride, int t, int j) {
    return (int)((const IdxT *)idx)[(int64_t)t * stride + j];
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace r3
