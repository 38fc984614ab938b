// Device-side helpers shared by the libzq kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zq {

typedef _Float16 half_t;
typedef int32_t int32x4 __attribute__((ext_vector_type(4)));
typedef int32_t int32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}

// The symmetric quantizer of App. A.2 for one value: v * inv, rounded half to
// even (v_rndne_f32), clamped to +-qmax.  One fp32 multiply, no fused add.
__device__ __forceinline__ int quant_code(float v, float inv, float qmax) {
    float t = v * inv;
    float r = rintf(t);
    r = fminf(fmaxf(r, -qmax), qmax);
    return (int)r;
}

// scale = fl32(a / qmax), inv = fl32(qmax / a); an all-zero block gets 0 / 0.
__device__ __forceinline__ void quant_scales(float a, float qmax, float &scale, float &inv) {
    if (a > 0.0f) {
        scale = a / qmax;
        inv = qmax / a;
    } else {
        scale = 0.0f;
        inv = 0.0f;
    }
}

__device__ __forceinline__ uint32_t pack4_i8(int a, int b, int c, int d) {
    return (uint32_t)(a & 0xff) | ((uint32_t)(b & 0xff) << 8) | ((uint32_t)(c & 0xff) << 16) |
           ((uint32_t)(d & 0xff) << 24);
}

// Workgroup barrier for kernels that keep asynchronous global->LDS loads in flight across it.
// __syncthreads() carries a fence that drains every outstanding vector-memory operation
// (s_waitcnt vmcnt(0)), which would serialise the load pipeline; here only LDS traffic is
// drained, and the "memory" clobber keeps the compiler from moving accesses across the barrier.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace zq
