// Measurement probes: the two ceilings the GeMM kernels are read against on the installed part.
// They are not steps of the quantized layer; bench.py runs them so that every roofline fraction can
// be stated twice, against the datasheet peak and against what the hardware sustains:
//   * a read-only stream over a buffer far larger than the caches (HBM read ceiling), and
//   * back-to-back v_mfma_i32_32x32x32_i8 on register operands taken from caller-supplied bytes
//     (matrix-core ceiling; it depends on the operand bytes, because the chip lowers its clock under
//     the power a toggling data path draws), and
//   * the same matrix-core stream fed the way the 256x256 tile of the tiled GeMM feeds it: fragments
//     read from LDS for every k step and operand stages arriving global -> LDS, with no barrier, no
//     prologue and no epilogue (what the part sustains once the operand movement shares the power
//     budget: the ceiling of that tile design, not of a particular kernel).
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

// Eight waves per workgroup, one workgroup per compute unit (128 KB of LDS), every wave the 128 x 64 wave
// tile of the tiled GeMM: eight accumulators, per k step six 16-byte fragment reads from LDS (two of one
// operand, four of the other) feeding eight MFMAs, and once per four k steps eight 1 KB direct loads
// global -> LDS per wave (together the 64 KB of a 256 x 256 x 128-byte stage) from a 2 MB window that
// stays in the L2.  The loads of a stage are waited for one stage later; nothing orders the waves, so the
// products are meaningless: only the traffic and the instruction mix are those of the GeMM.
typedef __attribute__((address_space(3))) void probe_lds_void;
__global__ __launch_bounds__(512, 1) void probe_mfma_i8_tile_traffic_kernel(const uint8_t *__restrict__ src, int iters,
                                                                            int32x4 *__restrict__ sink) {
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ __attribute__((aligned(16))) uint8_t probe_smem[];
    constexpr int kWindow = 2 << 20;
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    for (int i = threadIdx.x; i < 131072 / 16; i += 512)
        reinterpret_cast<int32x4 *>(probe_smem)[i] =
            reinterpret_cast<const int32x4 *>(src)[(blockIdx.x * 8192 + i) & (kWindow / 16 - 1)];
    __syncthreads();
    int32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0;
    int32x4 a[2][2], b[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < 2; ++i) a[s][i] = reinterpret_cast<int32x4 *>(probe_smem)[wave * 64 + lane + 512 * (s * 6 + i)];
#pragma unroll
        for (int i = 0; i < 4; ++i) b[s][i] = reinterpret_cast<int32x4 *>(probe_smem)[wave * 64 + lane + 512 * (s * 6 + 2 + i)];
    }
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(src), 0, kWindow, 0x00020000u);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            // fragment-shaped reads: 64 lanes x 16 contiguous bytes, six different kilobytes per k step,
            // all inside the first 72 KB of the 128 KB (offsets below 65536 + 5120 + 1024)
            const int base = ((it * 4 + ks) * 6 * 1024 + wave * 12288) & 0xffff;
#pragma unroll
            for (int i = 0; i < 2; ++i)
                a[nxt][i] = *reinterpret_cast<const int32x4 *>(probe_smem + base + i * 1024 + lane * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                b[nxt][i] = *reinterpret_cast<const int32x4 *>(probe_smem + base + (2 + i) * 1024 + lane * 16);
            if (ks == 3) {
                __builtin_amdgcn_s_waitcnt(0x0f70);          // vmcnt(0): the loads issued one stage ago
#pragma unroll
                for (int l = 0; l < 8; ++l) {
                    const int off = (((it * 8 + wave) * 8 + l) * 1024 + lane * 16) & (kWindow - 1);
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rs, (probe_lds_void *)(probe_smem + ((it & 1) * 65536 + (wave * 8 + l) * 1024)), 16, off, 0, 0, 0);
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i * 4 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[cur][i], b[cur][j], acc[i * 4 + j], 0, 0, 0);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);                      // no load may outlive the workgroup's LDS
    __syncthreads();
    int32x4 r = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) r[e & 3] += acc[i][e];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < 2; ++i) r += a[s][i];
#pragma unroll
        for (int i = 0; i < 4; ++i) r += b[s][i];
    }
    sink[(size_t)blockIdx.x * 512 + threadIdx.x] = r;
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

zq_status zq_probe_mfma_i8_tile_traffic(const void *source, size_t source_bytes, int blocks, int iters, void *sink,
                                        zq_stream stream) {
    if (source == nullptr || sink == nullptr) return ZQ_ERR_NULL;
    if (source_bytes < (2u << 20) || blocks <= 0 || blocks > 65536 || iters <= 0) return ZQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(source) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 15u) != 0)
        return ZQ_ERR_ALIGN;
    static std::atomic<uint64_t> configured{0};
    const void *kernel = reinterpret_cast<const void *>(&zq::probe_mfma_i8_tile_traffic_kernel);
    if (zq::ensure_dynamic_lds(kernel, 131072, configured) != hipSuccess) return ZQ_ERR_HIP;
    hipLaunchKernelGGL(zq::probe_mfma_i8_tile_traffic_kernel, dim3(blocks), dim3(512), 131072,
                       reinterpret_cast<hipStream_t>(stream), reinterpret_cast<const uint8_t *>(source), iters,
                       reinterpret_cast<zq::int32x4 *>(sink));
    return hipGetLastError() == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

}  // extern "C"
