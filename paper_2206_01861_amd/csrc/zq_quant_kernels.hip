// Quantization kernels of libzq (gfx950):
//   * group-wise weight quantization, INT8 and packed INT4 (Sec. 4.1, App. A.2)
//   * LayerNorm / bias+GeLU / identity fused with token-wise INT8 quantization
//     (Sec. 4.1; Sec. 4.3 and App. D, "Operation Fusion for Token-wise
//     Activation Quantization").
// All of them are bound by HBM traffic: reads are 16-byte vectors, coalesced
// along the row; a row is read once and stays in registers between the
// reduction that finds its scale and the pass that emits its codes.
#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

// ---------------------------------------------------------------------------
// Row front-ends.  A row is handled by TPR threads (one wave, or the whole
// 256-thread workgroup), each holding VPT vectors of 8 elements in registers.
// ---------------------------------------------------------------------------

template <int TPR>
__device__ __forceinline__ float row_sum(float v, float *lds) {
    v = wave_sum(v);
    if (TPR > kWave) {
        const int w = threadIdx.x / kWave;
        __syncthreads();
        if ((threadIdx.x % kWave) == 0) lds[w] = v;
        __syncthreads();
        v = lds[0] + lds[1] + lds[2] + lds[3];
    }
    return v;
}

template <int TPR>
__device__ __forceinline__ float row_max(float v, float *lds) {
    v = wave_max(v);
    if (TPR > kWave) {
        const int w = threadIdx.x / kWave;
        __syncthreads();
        if ((threadIdx.x % kWave) == 0) lds[w] = v;
        __syncthreads();
        v = fmaxf(fmaxf(lds[0], lds[1]), fmaxf(lds[2], lds[3]));
    }
    return v;
}

template <int OP, int TPR, int VPT>
__global__ __launch_bounds__(256) void rowquant_kernel(const half8 *__restrict__ in, const half8 *__restrict__ p0,
                                                       const half8 *__restrict__ p1, float eps, int M, int K,
                                                       int8_t *__restrict__ xq, float *__restrict__ s_tok,
                                                       void *__restrict__ y_out, int y_dtype) {
    __shared__ float lds[4];
    constexpr int RPB = 256 / TPR;
    const int t = threadIdx.x % TPR;
    const int row = blockIdx.x * RPB + threadIdx.x / TPR;
    if (TPR <= kWave && row >= M) return;   // whole waves leave together; no block barrier is used
    const int nvec = K >> 3;
    const half8 *rin = in + (size_t)row * nvec;

    constexpr bool kGelu = (OP == kOpGeluErf || OP == kOpGeluTanh);
    // Every load of the row and (for up to four vectors per thread) of its parameters is issued before
    // the first result is waited for: vectors past the end of the row read vector 0 instead of being
    // skipped, so that no branch separates the loads and one memory round trip covers them all.
    constexpr bool kPre = (VPT <= 4) && (OP == kOpLayerNorm || kGelu);
    bool ok[VPT];
    int idc[VPT];
    uint32x4_t raw[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int idx = i * TPR + t;
        ok[i] = idx < nvec;
        idc[i] = ok[i] ? idx : 0;
        raw[i] = __builtin_bit_cast(uint32x4_t, rin[idc[i]]);
    }
    uint32x4_t pa[kPre ? VPT : 1], pb[kPre ? VPT : 1];
    if (kPre && OP == kOpLayerNorm) {
        // gamma is always there; without beta, gamma is loaded a second time (a cache hit) and not
        // used, which keeps the loads free of branches
        const half8 *q1 = p1 != nullptr ? p1 : p0;
#pragma unroll
        for (int i = 0; i < (kPre ? VPT : 0); ++i) {
            pa[i] = __builtin_bit_cast(uint32x4_t, p0[idc[i]]);
            pb[i] = __builtin_bit_cast(uint32x4_t, q1[idc[i]]);
        }
    } else if (kPre && p0 != nullptr) {
#pragma unroll
        for (int i = 0; i < (kPre ? VPT : 0); ++i) pa[i] = __builtin_bit_cast(uint32x4_t, p0[idc[i]]);
    }

    float v[VPT][8];
    if (!kGelu) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const half8 h = __builtin_bit_cast(half8, raw[i]);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[i][e] = ok[i] ? (float)h[e] : 0.0f;
        }
    }

    if (OP == kOpLayerNorm) {
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < VPT; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[i][e];
        const float mean = row_sum<TPR>(s, lds) / (float)K;
        float ss = 0.0f;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            if (ok[i]) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float d = v[i][e] - mean;
                    ss += d * d;
                }
            }
        }
        const float var = row_sum<TPR>(ss, lds) / (float)K;
        const float rstd = 1.0f / sqrtf(var + eps);
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            if (ok[i]) {
                const half8 g = kPre ? __builtin_bit_cast(half8, pa[kPre ? i : 0]) : p0[idc[i]];
                if (p1 != nullptr) {
                    const half8 b = kPre ? __builtin_bit_cast(half8, pb[kPre ? i : 0]) : p1[idc[i]];
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[i][e] = (v[i][e] - mean) * rstd * (float)g[e] + (float)b[e];
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[i][e] = (v[i][e] - mean) * rstd * (float)g[e];
                }
            }
        }
    } else if (kGelu) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            if (ok[i]) {
                if (p0 != nullptr) {
                    const uint32x4_t b = kPre ? pa[kPre ? i : 0] : __builtin_bit_cast(uint32x4_t, p0[idc[i]]);
#pragma unroll
                    for (int d = 0; d < 4; ++d) add2_f16_f32(raw[i][d], b[d], v[i][2 * d], v[i][2 * d + 1]);
                } else {
                    const half8 h = __builtin_bit_cast(half8, raw[i]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[i][e] = (float)h[e];
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) v[i][e] = (OP == kOpGeluErf) ? gelu_erf(v[i][e]) : gelu_tanh(v[i][e]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[i][e] = 0.0f;
            }
        }
    }

    // Token-wise scale (Sec. 4.1): absmax of the row, from registers.
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < VPT; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf(v[i][e]));
    a = row_max<TPR>(a, lds);
    float scale, inv;
    quant_scales(a, 127.0f, scale, inv);
    if (t == 0) s_tok[row] = scale;

    uint2 *rq = reinterpret_cast<uint2 *>(xq + (size_t)row * K);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int idx = i * TPR + t;
        if (ok[i]) {
            if (y_out != nullptr) {
                if (y_dtype == 1) {
                    float4 *yo = reinterpret_cast<float4 *>(reinterpret_cast<float *>(y_out) + (size_t)row * K) + 2 * idx;
                    yo[0] = make_float4(v[i][0], v[i][1], v[i][2], v[i][3]);
                    yo[1] = make_float4(v[i][4], v[i][5], v[i][6], v[i][7]);
                } else {
                    half8 h;
#pragma unroll
                    for (int e = 0; e < 8; ++e) h[e] = (half_t)v[i][e];
                    reinterpret_cast<half8 *>(reinterpret_cast<half_t *>(y_out) + (size_t)row * K)[idx] = h;
                }
            }
            uint32_t q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) q[e] = quant_code_bits(v[i][e], inv);
            rq[idx] = make_uint2(pack4_code_bits(q[0], q[1], q[2], q[3]), pack4_code_bits(q[4], q[5], q[6], q[7]));
        }
    }
}

template <int OP, int TPR, int VPT>
static hipError_t launch_rq(const void *in, const void *p0, const void *p1, float eps, int M, int K, int8_t *xq,
                            float *s_tok, void *y_out, int y_dtype, hipStream_t st) {
    constexpr int RPB = 256 / TPR;
    const int blocks = (M + RPB - 1) / RPB;
    hipLaunchKernelGGL((rowquant_kernel<OP, TPR, VPT>), dim3(blocks), dim3(256), 0, st,
                       reinterpret_cast<const half8 *>(in), reinterpret_cast<const half8 *>(p0),
                       reinterpret_cast<const half8 *>(p1), eps, M, K, xq, s_tok, y_out, y_dtype);
    return hipGetLastError();
}

template <int OP>
static hipError_t launch_rq_op(const void *in, const void *p0, const void *p1, float eps, int M, int K, int8_t *xq,
                               float *s_tok, void *y_out, int y_dtype, hipStream_t st) {
    const int nvec = K / 8;
#define ZQ_RQ(TPR, VPT) return launch_rq<OP, TPR, VPT>(in, p0, p1, eps, M, K, xq, s_tok, y_out, y_dtype, st)
    // Short rows: one wave per row, four rows per workgroup.
    if (nvec <= 64 * 1) ZQ_RQ(64, 1);
    if (nvec <= 64 * 2) ZQ_RQ(64, 2);
    // Longer rows: the whole workgroup shares one row.
    if (nvec <= 256 * 1) ZQ_RQ(256, 1);
    if (nvec <= 256 * 2) ZQ_RQ(256, 2);
    if (nvec <= 256 * 3) ZQ_RQ(256, 3);
    if (nvec <= 256 * 4) ZQ_RQ(256, 4);
    if (nvec <= 256 * 6) ZQ_RQ(256, 6);
    if (nvec <= 256 * 8) ZQ_RQ(256, 8);
    if (nvec <= 256 * 12) ZQ_RQ(256, 12);
    if (nvec <= 256 * 16) ZQ_RQ(256, 16);
#undef ZQ_RQ
    return hipErrorInvalidValue;
}

hipError_t launch_rowquant(RowOp op, const void *in, const void *p0, const void *p1, float eps, int M, int K,
                           int8_t *xq, float *s_tok, void *y_out, int y_dtype, hipStream_t st) {
    switch (op) {
        case kOpLayerNorm: return launch_rq_op<kOpLayerNorm>(in, p0, p1, eps, M, K, xq, s_tok, y_out, y_dtype, st);
        case kOpGeluErf: return launch_rq_op<kOpGeluErf>(in, p0, p1, eps, M, K, xq, s_tok, y_out, y_dtype, st);
        case kOpGeluTanh: return launch_rq_op<kOpGeluTanh>(in, p0, p1, eps, M, K, xq, s_tok, y_out, y_dtype, st);
        case kOpIdentity: return launch_rq_op<kOpIdentity>(in, p0, p1, eps, M, K, xq, s_tok, y_out, y_dtype, st);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------
// Stand-alone dequantization of an INT32 accumulator tensor: the separate
// kernel of the unfused pipeline (Fig. 2, left) that the GeMM epilogue
// replaces (fp32 arithmetic, one FP16 rounding).
// One thread per four consecutive columns (a group holds a multiple of 16).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dequant_kernel(const int32x4 *__restrict__ acc, const float *__restrict__ s_tok,
                                                      const float *__restrict__ s_w, int gs,
                                                      const half_t *__restrict__ bias, int M, int N,
                                                      half4 *__restrict__ out) {
    const int nq = N >> 2;
    const long total = (long)M * nq;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int m = (int)(i / nq);
        const int n = (int)(i - (long)m * nq) * 4;
        const int32x4 v = acc[i];
        const float sc = s_tok[m] * s_w[n / gs];
        half4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float f = (float)v[e] * sc;
            if (bias != nullptr) f += (float)bias[n + e];
            o[e] = (half_t)f;
        }
        out[i] = o;
    }
}

hipError_t launch_dequant(const int32_t *acc, const float *s_tok, const float *s_w, int groups, const void *bias, int M,
                          int N, void *out, hipStream_t st) {
    const long total = (long)M * (N / 4);
    long blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(dequant_kernel, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<const int32x4 *>(acc),
                       s_tok, s_w, N / groups, reinterpret_cast<const half_t *>(bias), M, N,
                       reinterpret_cast<half4 *>(out));
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Group-wise weight quantization.  A group is a contiguous chunk of gs*K fp16
// values.  Four launches: clear, absmax (integer atomic max on the fp32 bit
// pattern, exact and order independent), quantize, and turn absmax into the
// scale in place.  s_w doubles as the absmax scratch, so nothing is allocated.
// ---------------------------------------------------------------------------

__global__ void wq_clear_kernel(uint32_t *amax_bits, int groups) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < groups) amax_bits[i] = 0u;
}

__global__ __launch_bounds__(256) void wq_absmax_kernel(const uint4 *__restrict__ w, long chunk_vecs, long slice_vecs,
                                                        uint32_t *__restrict__ amax_bits) {
    __shared__ uint32_t lds[4];
    const int g = blockIdx.y;
    const long lo = (long)blockIdx.x * slice_vecs;
    long hi = lo + slice_vecs;
    if (hi > chunk_vecs) hi = chunk_vecs;
    const uint4 *base = w + (long)g * chunk_vecs;
    // |fp16| compares like its 15-bit pattern; keep the maximum pattern.
    uint32_t m = 0;
    for (long i = lo + threadIdx.x; i < hi; i += 256) {
        uint4 u = base[i];
        uint32_t d[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t a0 = d[e] & 0x7fffu, a1 = (d[e] >> 16) & 0x7fffu;
            m = a0 > m ? a0 : m;
            m = a1 > m ? a1 : m;
        }
    }
    m = wave_max_u32(m);
    if ((threadIdx.x % kWave) == 0) lds[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t r = lds[0];
        r = lds[1] > r ? lds[1] : r;
        r = lds[2] > r ? lds[2] : r;
        r = lds[3] > r ? lds[3] : r;
        union { uint16_t u; half_t h; } cv;
        cv.u = (uint16_t)r;
        const float a = (float)cv.h;
        atomicMax(amax_bits + g, __float_as_uint(a));   // non-negative floats order like their bits
    }
}

template <int BITS>
__global__ __launch_bounds__(256) void wq_quant_kernel(const half8 *__restrict__ w, long chunk_vecs, long slice_vecs,
                                                       const float *__restrict__ amax, void *__restrict__ wq) {
    const int g = blockIdx.y;
    const long lo = (long)blockIdx.x * slice_vecs;
    long hi = lo + slice_vecs;
    if (hi > chunk_vecs) hi = chunk_vecs;
    const float qmax = (BITS == 8) ? 127.0f : 7.0f;
    float scale, inv;
    quant_scales(amax[g], qmax, scale, inv);
    const long gbase = (long)g * chunk_vecs;
    for (long i = lo + threadIdx.x; i < hi; i += 256) {
        half8 h = w[gbase + i];
        uint32_t q[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = quant_code_bits((float)h[e], inv);
        if (BITS == 8) {
            reinterpret_cast<uint2 *>(wq)[gbase + i] =
                make_uint2(pack4_code_bits(q[0], q[1], q[2], q[3]), pack4_code_bits(q[4], q[5], q[6], q[7]));
        } else {
            uint32_t p = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) p |= (q[e] & 0xfu) << (4 * e);   // even k in the low nibble
            reinterpret_cast<uint32_t *>(wq)[gbase + i] = p;
        }
    }
}

__global__ void wq_finalize_kernel(float *s_w, int groups, float qmax) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < groups) {
        float scale, inv;
        quant_scales(s_w[i], qmax, scale, inv);
        s_w[i] = scale;
    }
}

hipError_t launch_weight_quant(const void *w, int N, int K, int groups, int bits, void *wq, float *s_w,
                               hipStream_t st) {
    const long chunk_vecs = (long)(N / groups) * K / 8;
    // enough slices per group to put a few thousand workgroups in flight
    long P = (4096 + groups - 1) / groups;
    const long max_p = (chunk_vecs + 255) / 256;
    if (P > max_p) P = max_p;
    if (P < 1) P = 1;
    const long slice_vecs = (chunk_vecs + P - 1) / P;
    const dim3 grid((unsigned)P, (unsigned)groups);
    const int cb = (groups + 255) / 256;
    hipLaunchKernelGGL(wq_clear_kernel, dim3(cb), dim3(256), 0, st, reinterpret_cast<uint32_t *>(s_w), groups);
    hipLaunchKernelGGL(wq_absmax_kernel, grid, dim3(256), 0, st, reinterpret_cast<const uint4 *>(w), chunk_vecs,
                       slice_vecs, reinterpret_cast<uint32_t *>(s_w));
    if (bits == 8)
        hipLaunchKernelGGL(wq_quant_kernel<8>, grid, dim3(256), 0, st, reinterpret_cast<const half8 *>(w), chunk_vecs,
                           slice_vecs, s_w, wq);
    else
        hipLaunchKernelGGL(wq_quant_kernel<4>, grid, dim3(256), 0, st, reinterpret_cast<const half8 *>(w), chunk_vecs,
                           slice_vecs, s_w, wq);
    hipLaunchKernelGGL(wq_finalize_kernel, dim3(cb), dim3(256), 0, st, s_w, groups, bits == 8 ? 127.0f : 7.0f);
    return hipGetLastError();
}

}  // namespace zq
