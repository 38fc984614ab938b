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

typedef float float32x4 __attribute__((ext_vector_type(4)));
typedef float float32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t uint32x4_t __attribute__((ext_vector_type(4)));

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

// The symmetric quantizer of App. A.2 for one value: fl32(v * inv) rounded half to even.  The
// rounding is done by adding 1.5 * 2^23: the sum is rounded to an integer by the adder (round to
// nearest even, the same rounding as v_rndne_f32) and its low mantissa bits hold that integer in
// two's complement, so the code is the low byte of the result and no float->int conversion is
// needed.  No clamp: |v| <= absmax of its block and inv = fl32(qmax / absmax), so
// |fl32(v * inv)| <= qmax * (1 + 2^-23) and rounds to at most qmax.  The product and the sum
// stay two separately rounded operations (no fused multiply-add), as the definition has them.
__device__ __forceinline__ uint32_t quant_code_bits(float v, float inv) {
#pragma clang fp contract(off)
    const float t = v * inv;
    const float r = t + 12582912.0f;
    return __float_as_uint(r);
}

// Low bytes of four quant_code_bits() results -> one dword, first value in the low byte.
__device__ __forceinline__ uint32_t pack4_code_bits(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    const uint32_t lo = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);   // a.b0, b.b0, 0, 0
    const uint32_t hi = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
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

// GeLU, erf form: u * Phi(u) = max(u, 0) - |u| * h with h = erfc(|u| / sqrt2) / 2 from the rational
// approximation of Abramowitz & Stegun 7.1.26 (absolute error of erf below 1.5e-7, i.e. below fp32
// resolution of Phi); going through erfc keeps the relative accuracy of the negative tail.  The
// constants carry the factors 1/sqrt2, 1/2 and log2(e).  About a third of the VALU work of the
// library erff, which otherwise makes this memory-bound kernel compute-bound.
__device__ __forceinline__ float gelu_erf(float u) {
    const float a = fabsf(u);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, a, 1.0f));
    // The leading coefficient lives in a register of its own (the asm has no inputs, so the
    // compiler keeps one copy): the first Horner step is then one multiply-add with one literal
    // instead of a move and a multiply-accumulate.
    float c5;
    asm("v_mov_b32 %0, 0x3f07dc22" : "=v"(c5));       // 0.5 * 1.061405429
    float p = fmaf(t, c5, 0.5f * -1.453152027f);
    p = fmaf(t, p, 0.5f * 1.421413741f);
    p = fmaf(t, p, 0.5f * -0.284496736f);
    p = fmaf(t, p, 0.5f * 0.254829592f);
    const float w = u * 0.84932180028801904272f;      // sqrt(log2(e) / 2): exp(-u^2 / 2) = 2^(-w^2)
    const float e = __builtin_amdgcn_exp2f(-(w * w));
    const float h = (p * t) * e;
    float pos;                                        // max(u, 0) in one instruction (no canonicalising copy)
    asm("v_max_f32 %0, 0, %1" : "=v"(pos) : "v"(u));
    return fmaf(-a, h, pos);
}

// GeLU, tanh form: 0.5 u (1 + tanh(v)) = u * (1 - 1 / (1 + exp(2v))).
__device__ __forceinline__ float gelu_tanh(float u) {
    const float c = 0.79788456080286535588f;
    const float v = c * fmaf(0.044715f * u * u, u, u);
    const float e = __builtin_amdgcn_exp2f(v * (2.0f * 1.44269504088896340736f));
    return u * (1.0f - __builtin_amdgcn_rcpf(1.0f + e));
}

// Eight INT8 codes (two dwords, lowest byte first) -> eight FP16 values, exactly.  A code byte with
// its sign bit flipped is code + 128 as an unsigned byte u; under the high byte 0x64 it reads as
// the FP16 number 1024 + u (the FP16 spacing between 1024 and 2048 is 1), and subtracting 1152
// leaves the code.  Two XORs, four byte permutes and four packed FP16 subtractions.
__device__ __forceinline__ half8 cvt8_i8_f16(uint32_t lo, uint32_t hi) {
    const uint32_t ul = lo ^ 0x80808080u, uh = hi ^ 0x80808080u;
    const uint32_t k = 0x64646464u;
    uint32x4_t d;
    d[0] = __builtin_amdgcn_perm(k, ul, 0x04010400u);
    d[1] = __builtin_amdgcn_perm(k, ul, 0x04030402u);
    d[2] = __builtin_amdgcn_perm(k, uh, 0x04010400u);
    d[3] = __builtin_amdgcn_perm(k, uh, 0x04030402u);
    half8 h = __builtin_bit_cast(half8, d);
    const half_t bias = (half_t)1152.0f;
    return h - half8{bias, bias, bias, bias, bias, bias, bias, bias};
}

// Activation fused into a GeMM epilogue: 0 none, 1 GeLU (erf form), 2 GeLU (tanh form).
__device__ __forceinline__ float apply_activation(float f, int act) {
    if (act == 1) return gelu_erf(f);
    if (act == 2) return gelu_tanh(f);
    return f;
}

// The same over N values at once.  The choice is made once, outside the loop over the values, so each
// branch is straight-line code whose N dependency chains (one reciprocal and one exponential each)
// the compiler can interleave; with the choice inside, every value ran its chain alone.
template <int N>
__device__ __forceinline__ void apply_activation_n(float (&f)[N], int act) {
    if (act == 1) {
#pragma unroll
        for (int e = 0; e < N; ++e) f[e] = gelu_erf(f[e]);
    } else if (act == 2) {
#pragma unroll
        for (int e = 0; e < N; ++e) f[e] = gelu_tanh(f[e]);
    }
}

// Workgroup barrier for kernels that keep asynchronous global->LDS loads in flight across it.
// __syncthreads() carries a fence that drains every outstanding vector-memory operation
// (s_waitcnt vmcnt(0)), which would serialise the load pipeline; here only LDS traffic is
// drained, and the "memory" clobber keeps the compiler from moving accesses across the barrier.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace zq
