// FP16 activations x INT8 group-wise weights (the W8A16 setting of Sec. 5:
// the QKV GeMM of the largest model keeps its FP16 input; App. A.2 quantizer
// for the weights), with the weight-scale epilogue
//   out[m,n] = fp16( (sum_k x[m,k] * wq[n,k]) * s_w[n / (N/groups)] + bias[n] ).
// The INT8 codes are converted to FP16 in registers (exact: |code| <= 127) and
// multiplied on the FP16 matrix cores with fp32 accumulation.
//
// This file holds the schedule that takes every legal shape: one wavefront per
// 16x16 output tile, operands straight from global memory,
// v_mfma_f32_16x16x32_f16.  Token counts up to 64 with K a multiple of 256 go
// to the weight-streaming schedule instead (zq_gemm_skinny.hip).
#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

__global__ __launch_bounds__(256) void gemm_a16_simple_kernel(const half_t *__restrict__ x,
                                                              const int8_t *__restrict__ wq,
                                                              const float *__restrict__ s_w, int gs,
                                                              const half_t *__restrict__ bias, int M, int N, int K,
                                                              half_t *__restrict__ out) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int n0 = (blockIdx.x * 4 + wave) * 16;
    const int m0 = blockIdx.y * 16;
    if (n0 >= N) return;
    const int r = lane % 16;
    const int kc = (lane / 16) * 8;           // this lane's 8 values of each 32-deep step
    int mrow = m0 + r;
    if (mrow > M - 1) mrow = M - 1;           // rows past M are computed from a valid row and never stored
    const half_t *xrow = x + (size_t)mrow * K;
    const int8_t *wrow = wq + (size_t)(n0 + r) * K;

    float32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int k0 = 0; k0 < K; k0 += 32) {
        const int k = k0 + kc;
        half8 a = {0, 0, 0, 0, 0, 0, 0, 0}, b = {0, 0, 0, 0, 0, 0, 0, 0};
        if (k < K) {                           // K % 16 == 0, so a slice of 8 is all inside or all outside
            b = *reinterpret_cast<const half8 *>(xrow + k);
            const uint2 p = *reinterpret_cast<const uint2 *>(wrow + k);
            a = cvt8_i8_f16(p.x, p.y);
        }
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc, 0, 0, 0);
    }

    // Accumulator layout: register v of lane l is tile row 4*(l/16)+v of the first operand (a weight
    // row = output column) and column l%16 of the second (a token).
    const int m = m0 + r;
    if (m >= M) return;
    const int n = n0 + 4 * (lane / 16);
    const float sw = s_w[n / gs];              // four consecutive columns never straddle a group (gs % 16 == 0)
    half4 o;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        float f = acc[v] * sw;
        if (bias != nullptr) f += (float)bias[n + v];
        o[v] = (half_t)f;
    }
    *reinterpret_cast<half4 *>(out + (size_t)m * N + n) = o;
#endif
}

hipError_t launch_gemm_a16_simple(const A16Args &a, hipStream_t st) {
    const dim3 grid((a.N / 16 + 3) / 4, (a.M + 15) / 16);
    hipLaunchKernelGGL(gemm_a16_simple_kernel, grid, dim3(256), 0, st, reinterpret_cast<const half_t *>(a.x),
                       reinterpret_cast<const int8_t *>(a.wq), a.s_w, a.N / a.groups,
                       reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K, reinterpret_cast<half_t *>(a.out));
    return hipGetLastError();
}

}  // namespace zq
