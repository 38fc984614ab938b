// Measurement probes: the two ceilings the GeMM kernels are read against on the installed part.
// They are not steps of the quantized layer; bench.py runs them so that every roofline fraction can
// be stated twice, against the datasheet peak and against what the hardware sustains:
//   * a read-only stream over a buffer far larger than the caches (HBM read ceiling), and
//   * back-to-back v_mfma_i32_32x32x32_i8 on register operands taken from caller-supplied bytes
//     (matrix-core ceiling; it depends on the operand bytes, because the chip lowers its clock under
//     the power a toggling data path draws).
#include "../../include/zq_probe.h"
#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

// Every thread reads 16-byte pieces with a grid stride, four independent loads per round; the sum is
// stored only under a condition that random data never meets, so the loads cannot be optimised away.
__global__ __launch_bounds__(256) void probe_read_stream_kernel(const int32x4 *__restrict__ in, size_t n,
                                                                int32x4 *__restrict__ sink) {
    int32x4 r = {0, 0, 0, 0};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const int32x4 a = in[i], b = in[i + stride], c = in[i + 2 * stride], d = in[i + 3 * stride];
        r += a + b + c + d;
    }
    for (; i < n; i += stride) r += in[i];
    if (r[0] == 0x12345678 && r[1] == 0x0badf00d && r[2] == r[3]) sink[0] = r;
}

// One wave = the register tile of a 128 x 128 product: four fragments of each operand (the bytes come
// from `operands`, 128 bytes per thread), sixteen accumulators, `iters` rounds of sixteen MFMAs.
__global__ __launch_bounds__(256) void probe_mfma_i8_kernel(const int32x4 *__restrict__ operands, int iters,
                                                            int32x4 *__restrict__ sink) {
#if defined(__HIP_DEVICE_COMPILE__)
    int32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0;
    int32x4 a[4], b[4];
    const size_t t = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = operands[t + i];
        b[i] = operands[t + 4 + i];
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
    }
    int32x4 r = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) r[e & 3] += acc[i][e];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
#endif
}

}  // namespace zq

extern "C" {

zq_status zq_probe_read_stream(const void *buf, size_t bytes, void *sink, zq_stream stream) {
    if (buf == nullptr || sink == nullptr) return ZQ_ERR_NULL;
    if (bytes < 16 || (bytes % 16) != 0) return ZQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 15u) != 0)
        return ZQ_ERR_ALIGN;
    const int blocks = zq::compute_units() * 8;
    hipLaunchKernelGGL(zq::probe_read_stream_kernel, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<const zq::int32x4 *>(buf), bytes / 16, reinterpret_cast<zq::int32x4 *>(sink));
    return hipGetLastError() == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

zq_status zq_probe_mfma_i8(const void *operands, int blocks, int iters, void *sink, zq_stream stream) {
    if (operands == nullptr || sink == nullptr) return ZQ_ERR_NULL;
    if (blocks <= 0 || blocks > 65536 || iters <= 0) return ZQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(operands) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 15u) != 0)
        return ZQ_ERR_ALIGN;
    hipLaunchKernelGGL(zq::probe_mfma_i8_kernel, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<const zq::int32x4 *>(operands), iters, reinterpret_cast<zq::int32x4 *>(sink));
    return hipGetLastError() == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

}  // extern "C"
