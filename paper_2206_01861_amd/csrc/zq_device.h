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

// One cross-lane move on the data-parallel-primitive path (no LDS crossbar, a few cycles): every lane
// receives the value of the lane that CTRL names within its row of 16.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// The value that lane `lane` holds, as a scalar.
__device__ __forceinline__ float read_lane(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
constexpr int kDppXor1 = 0xB1;          // quad_perm:[1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // row_half_mirror: lane i of each 8 <- lane 7 - i
constexpr int kDppMirror = 0x140;       // row_mirror: lane i of each 16 <- lane 15 - i

// Reductions over the 64 lanes of a wave; every lane must be active and every lane gets the result.
// Four steps inside each row of 16 lanes (after each, the lanes that have been combined hold the same
// bits, since both partners add or compare the same two values), then the four row results are read
// as scalars.  A butterfly of six ds_bpermute round trips is several hundred cycles of latency per
// reduction, which the row kernels (one short pass per row) cannot hide.
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_move<kDppXor1>(v));
    v = fmaxf(v, dpp_move<kDppXor2>(v));
    v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_move<kDppMirror>(v));
    const float r0 = read_lane(v, 0), r1 = read_lane(v, 16), r2 = read_lane(v, 32), r3 = read_lane(v, 48);
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    v += dpp_move<kDppMirror>(v);
    const float r0 = read_lane(v, 0), r1 = read_lane(v, 16), r2 = read_lane(v, 32), r3 = read_lane(v, 48);
    return (r0 + r1) + (r2 + r3);
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

// fl32(h) + fl32(b) for the two FP16 values held in each of the dwords hw and bw (low half -> lo).  One
// mixed-precision multiply-add per value, h * 1 + b with h and b read as FP16 and rounded once to fp32,
// which is the sum of the two exact conversions; it replaces two conversions and an addition.
__device__ __forceinline__ void add2_f16_f32(uint32_t hw, uint32_t bw, float &lo, float &hi) {
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,1]" : "=v"(lo) : "v"(hw), "v"(bw));
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,1] op_sel_hi:[1,0,1]" : "=v"(hi) : "v"(hw), "v"(bw));
}

// GeLU, erf form: u * Phi(u) = max(u, 0) - a * Phi(-a) with a = |u|, and Phi(-a) = 2^P(a) with P a degree-6
// polynomial: log2 Phi(-a) is smooth (close to a parabola), so a short polynomial in a reaches fp32
// resolution where a rational or erfc-style approximation needs a reciprocal on top of the exponential.
// P was fitted on [0, 5.6] to the exact log2 Phi(-a) (minimax of the error in a * Phi(-a), P(0) = -1
// kept exact so the relative error vanishes towards u = 0); beyond 5.6, where a * Phi(-a) < 6e-8, a is
// held at 5.6.  Error of the result evaluated in fp32: below 1.2e-7 absolute, below 1.5e-6 relative for
// |u| < 1.  Thirteen VALU cycles per value (six multiply-adds, a minimum, a maximum, one exponential
// at quarter rate, one multiply-add), against nineteen for Abramowitz & Stegun 7.1.26 with its reciprocal.
__device__ __forceinline__ float gelu_erf(float u) {
    float a;                                          // min(|u|, 5.6) in one instruction (fminf would first quiet |u|)
    asm("v_min_f32 %0, |%1|, %2" : "=v"(a) : "v"(u), "s"(5.6f));
    // The leading coefficient lives in a register of its own (the asm has no inputs, so the
    // compiler keeps one copy): the first Horner step is then one multiply-add with one literal
    // instead of a move and a multiply-accumulate.
    float c6;
    asm("v_mov_b32 %0, 0x37fb05d2" : "=v"(c6));       // 2.9924242e-05
    float p = fmaf(a, c6, -7.3987467e-04f);
    p = fmaf(a, p, 7.9774642e-03f);
    p = fmaf(a, p, -5.3238187e-02f);
    p = fmaf(a, p, -4.5891568e-01f);
    p = fmaf(a, p, -1.1511471f);
    p = fmaf(a, p, -1.0f);
    const float h = __builtin_amdgcn_exp2f(p);        // Phi(-a), 1e-8 .. 0.5
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
// drained.  The wait is emitted through the builtin so that the compiler's own wait-count
// bookkeeping sees it: with the wait hidden inside an asm statement the compiler assumed the LDS
// reads issued before the barrier could still be in flight after it, and made the matrix-core
// instructions that follow the barrier (on operands read long before) wait for the first reads
// issued after it.  The "memory" clobber keeps the compiler from moving accesses across the barrier.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0); vmcnt and expcnt untouched
    asm volatile("s_barrier" ::: "memory");
}

}  // namespace zq
