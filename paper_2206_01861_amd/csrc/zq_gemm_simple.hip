// Correctness-first INT8 GeMM with the dequantization epilogue (Sec. 4.3,
// App. D).  One wavefront owns one 16x16 output tile and feeds
// v_mfma_i32_16x16x64_i8 straight from global memory, so it accepts every
// legal shape (ragged M, K not a multiple of the tile depth).  The tuned
// schedules are checked against the oracle exactly like this one; this kernel
// is what the dispatcher falls back to when a shape fits none of them.
#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

// Sign-extend the eight nibbles of a packed word into two words of int8 codes
// in natural k order (low nibble = even k).
__device__ __forceinline__ void unpack8_plain(uint32_t p, uint32_t &lo4, uint32_t &hi4) {
    int c[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) c[e] = ((int)(p << (28 - 4 * e))) >> 28;
    lo4 = pack4_i8(c[0], c[1], c[2], c[3]);
    hi4 = pack4_i8(c[4], c[5], c[6], c[7]);
}

template <int WBITS>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const int8_t *__restrict__ xq, const float *__restrict__ s_tok,
                                                          const uint8_t *__restrict__ wq, const float *__restrict__ s_w,
                                                          int gs, const half_t *__restrict__ bias, int M, int N, int K,
                                                          half_t *__restrict__ out, int32_t *__restrict__ acc_out, int act) {
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int n0 = (blockIdx.x * 4 + wave) * 16;
    const int m0 = blockIdx.y * 16;
    if (n0 >= N) return;
    const int r = lane % 16;
    const int kc = (lane / 16) * 16;          // this lane's 16-byte slice of each 64-deep step
    int mrow = m0 + r;
    if (mrow > M - 1) mrow = M - 1;           // rows past M are computed from a valid row and never stored
    const int8_t *xrow = xq + (size_t)mrow * K;
    const size_t wrow_bytes = (WBITS == 8) ? (size_t)K : (size_t)(K / 2);
    const uint8_t *wrow = wq + (size_t)(n0 + r) * wrow_bytes;

    // The epilogue's operands first: their round trip then runs under the main loop.
    const int m_ld = (m0 + r < M) ? m0 + r : M - 1;
    const int n_ld = n0 + 4 * (lane / 16);
    const float sc = s_tok[m_ld] * s_w[n_ld / gs];   // four consecutive columns never straddle a group (gs % 16 == 0)
    half4 bv = {0, 0, 0, 0};
    if (bias != nullptr) bv = *reinterpret_cast<const half4 *>(bias + n_ld);

    auto load_step = [&](int k, int32x4 &a, int32x4 &b) __attribute__((always_inline)) {
        b = *reinterpret_cast<const int32x4 *>(xrow + k);
        if (WBITS == 8) {
            a = *reinterpret_cast<const int32x4 *>(wrow + k);
        } else {
            const uint2 p = *reinterpret_cast<const uint2 *>(wrow + k / 2);
            uint32_t w0, w1, w2, w3;
            unpack8_plain(p.x, w0, w1);
            unpack8_plain(p.y, w2, w3);
            a = int32x4{(int)w0, (int)w1, (int)w2, (int)w3};
        }
    };
    int32x4 acc = {0, 0, 0, 0};
    // Whole groups of four 64-deep steps.  The eight loads of a group are issued together and the
    // next group is requested before the current one is multiplied, so the loop costs about one
    // memory round trip per two groups instead of one per step.
    auto load_group = [&](int g, int32x4(&a)[4], int32x4(&b)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 4; ++u) load_step(g * 256 + 64 * u + kc, a[u], b[u]);
    };
    auto mfma_group = [&](const int32x4(&a)[4], const int32x4(&b)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u], b[u], acc, 0, 0, 0);
    };
    const int ng = K / 256;
    int32x4 a0[4], b0[4], a1[4], b1[4];
    if (ng > 0) load_group(0, a0, b0);
    for (int g = 0; g < ng; g += 2) {
        if (g + 1 < ng) load_group(g + 1, a1, b1);
        mfma_group(a0, b0);
        if (g + 1 < ng) {
            if (g + 2 < ng) load_group(g + 2, a0, b0);
            mfma_group(a1, b1);
        }
    }
    int k0 = ng * 256;
    for (; k0 < K; k0 += 64) {
        const int k = k0 + kc;
        int32x4 a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
        if (k < K) load_step(k, a, b);         // K % 16 == 0, so a slice is all inside or all outside
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc, 0, 0, 0);
    }

    // Accumulator layout: register v of lane l is tile row 4*(l/16)+v of the
    // first operand (a weight row = output column) and column l%16 of the
    // second (a token).
    const int m = m0 + r;
    if (m >= M) return;
    const int n = n0 + 4 * (lane / 16);
    float f[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) f[v] = (float)acc[v] * sc + (float)bv[v];   // bv is zero without a bias
    apply_activation_n<4>(f, act);
    half4 o;
#pragma unroll
    for (int v = 0; v < 4; ++v) o[v] = (half_t)f[v];
    *reinterpret_cast<half4 *>(out + (size_t)m * N + n) = o;
    if (acc_out != nullptr) *reinterpret_cast<int32x4 *>(acc_out + (size_t)m * N + n) = acc;
}

hipError_t launch_gemm_simple(const GemmArgs &a, hipStream_t st) {
    const dim3 grid((a.N / 16 + 3) / 4, (a.M + 15) / 16);
    const int gs = a.N / a.groups;
    if (a.w_bits == 8)
        hipLaunchKernelGGL(gemm_simple_kernel<8>, grid, dim3(256), 0, st, a.xq, a.s_tok,
                           reinterpret_cast<const uint8_t *>(a.wq), a.s_w, gs,
                           reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K,
                           reinterpret_cast<half_t *>(a.out), a.acc_out, a.act);
    else
        hipLaunchKernelGGL(gemm_simple_kernel<4>, grid, dim3(256), 0, st, a.xq, a.s_tok,
                           reinterpret_cast<const uint8_t *>(a.wq), a.s_w, gs,
                           reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K,
                           reinterpret_cast<half_t *>(a.out), a.acc_out, a.act);
    return hipGetLastError();
}

}  // namespace zq
