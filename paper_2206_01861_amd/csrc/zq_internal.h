// Host-side launcher declarations shared between the libzq translation units.
// Every launcher assumes its arguments were validated by the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace zq {

// Raise a kernel's dynamic LDS limit once per device (the attribute is per device; a process may
// drive several).  `done` is the caller's per-kernel bit mask of devices already configured.
inline hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes, std::atomic<uint64_t> &done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_relaxed) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    done.fetch_or(bit, std::memory_order_relaxed);
    return hipSuccess;
}

// Layout of a GeMM workspace (device memory the caller owns and zq_workspace_init() has zeroed):
//   [0, 256)            control words: [0] generation of the in-kernel output quantization,
//                       [1] workgroups of the running launch that have read their band,
//                       [2] threads whose bounded wait ran out
//   [256, +32 KB)       arrival counters of the strips a streaming schedule splits along K
//   [.., +4 MB)         exchange slots of the in-kernel output quantization (8 bytes per tile and row)
//   [kWsFixedBytes, ..) partial sums of the K-split schedules
// Every kernel leaves the first three parts ready for the next call; the parts never overlap, so
// calls of any kind and shape can share a workspace as long as they are ordered on one stream.
constexpr size_t kWsControlBytes = 256;
constexpr int kMaxSharedStrips = 8192;
constexpr int kMaxQuantSlots = 1 << 19;
constexpr size_t kWsCountersOffset = kWsControlBytes;
constexpr size_t kWsSlotsOffset = kWsCountersOffset + (size_t)kMaxSharedStrips * 4;
constexpr size_t kWsFixedBytes = kWsSlotsOffset + (size_t)kMaxQuantSlots * 8;
static_assert(kWsFixedBytes % 256 == 0, "the partial sums start on a 256-byte boundary");

inline unsigned *ws_control(void *ws) { return reinterpret_cast<unsigned *>(ws); }
inline unsigned *ws_counters(void *ws) { return reinterpret_cast<unsigned *>(static_cast<char *>(ws) + kWsCountersOffset); }
inline unsigned long long *ws_slots(void *ws) {
    return reinterpret_cast<unsigned long long *>(static_cast<char *>(ws) + kWsSlotsOffset);
}
inline void *ws_partials(void *ws) { return static_cast<char *>(ws) + kWsFixedBytes; }

// Compute units of the current device (256 when no device answers: the host-only queries still work).
int compute_units();

// Zero the fixed part of a workspace (a fill kernel, so the call may be captured into a graph).
hipError_t launch_workspace_init(void *ws, hipStream_t st);

enum RowOp { kOpLayerNorm = 0, kOpGeluErf = 1, kOpGeluTanh = 2, kOpIdentity = 3 };

// in fp16 [M,K]; p0 = gamma (LayerNorm) or bias (GeLU, nullable); p1 = beta (nullable).
hipError_t launch_rowquant(RowOp op, const void *in, const void *p0, const void *p1, float eps, int M, int K,
                           int8_t *xq, float *s_tok, void *y_out, int y_dtype, hipStream_t st);

// out fp16 [M,N] = acc * s_tok[row] * s_w[col group] + bias, the GeMM epilogue as a kernel of its own.
hipError_t launch_dequant(const int32_t *acc, const float *s_tok, const float *s_w, int groups, const void *bias, int M,
                          int N, void *out, hipStream_t st);

hipError_t launch_weight_quant(const void *w, int N, int K, int groups, int bits, void *wq, float *s_w,
                               hipStream_t st);

// GeMM schedules.  The order is part of the test/tuning hook of the C ABI.
enum GemmVariant {
    kGemmSimple = 0,      // one wave per 16x16 tile, operands from global; any legal shape
    kGemmTile128 = 1,     // 128x128 block tile, eight waves
    kGemmTile256 = 2,     // 256x256 block tile, eight waves
    kGemmSkinny = 3,      // M <= 128, K % 256 == 0: weight streaming, whole K in one workgroup
    kGemmSkinnySplitK = 4,// same, K also split across workgroups (needs workspace)
    kGemmTile256x128 = 5, // 256x128 block tile, four waves, two workgroups per CU
    kGemmTile256x192 = 6, // 256x192 block tile, eight waves: for grids that 256x256 tiles fill badly
    kGemmTileSplitK = 7,  // 128x128 block tile, K split over workgroups, epilogue in a second kernel (needs workspace)
    kGemmVariantCount = 8
};

struct GemmArgs {
    const int8_t *xq;
    const float *s_tok;
    const void *wq;       // int8 [N,K] or packed uint8 [N,K/2]
    const float *s_w;
    int groups;
    const void *bias;     // fp16 [N] or null
    int M, N, K;
    void *out;            // fp16 [M,N]
    int32_t *acc_out;     // nullable
    void *workspace;
    size_t workspace_bytes;
    int w_bits;           // 8 or 4
    int act;              // activation applied to acc*scale+bias before the FP16 rounding: 0 none, 1 GeLU erf, 2 GeLU tanh
    int8_t *q_out = nullptr;       // launch_gemm_tile_quant: int8 [M,N] codes of the output rows
    float *q_scale_out = nullptr;  //                         fp32 [M] their scales
};

// 128x128 tiles with a K split: how many splits pay for a shape (1 = none), the workspace they
// need, and the launch (two kernels).
int gemm_tile_splits(int M, int N, int K);
size_t gemm_tile_split_workspace(int M, int N, int K);
hipError_t launch_gemm_tile_splitk(const GemmArgs &a, hipStream_t st);

// Tiled GeMM that also quantizes its output rows token-wise inside the kernel (out may be null);
// needs a workspace of at least kWsFixedBytes.
bool gemm_tile_quant_supported(int M, int N, size_t workspace_bytes);
hipError_t launch_gemm_tile_quant(const GemmArgs &a, hipStream_t st);

// A caller-supplied cut of the streaming schedules for this shape, if one was registered.
bool tuned_stream_plan(int M, int N, int K, int w_bits, int *row_blocks, int *k_splits);

// FP16 activations x INT8 weights (W8A16).
struct A16Args {
    const void *x;        // fp16 [M,K]
    const void *wq;       // int8 [N,K]
    const float *s_w;
    int groups;
    const void *bias;     // fp16 [N] or null
    int M, N, K;
    void *out;            // fp16 [M,N]
    void *workspace;      // fp32 partials of the K split
    size_t workspace_bytes;
};
hipError_t launch_gemm_a16_simple(const A16Args &a, hipStream_t st);
hipError_t launch_gemm_a16_stream(const A16Args &a, bool allow_split, hipStream_t st);   // M <= 64, K % 256 == 0
size_t stream_a16_workspace_bytes(int M, int N, int K);                                   // of that schedule's K split
void stream_a16_plan(int M, int N, int K, bool allow_split, int *row_blocks, int *k_splits, int *consumers);
hipError_t launch_gemm_a16_tile(const A16Args &a, hipStream_t st);                       // any K the ABI accepts
int gemm_a16_tile_splits(int M, int N, int K);                                          // K splits that pay on tiles, 1 = none
size_t gemm_a16_tile_split_workspace(int M, int N, int K);                              // of its K split, 0 if none

bool gemm_variant_supports(int variant, int M, int N, int K, int w_bits, size_t workspace_bytes);
size_t gemm_variant_workspace(int variant, int M, int N, int K, int w_bits);
hipError_t launch_gemm(int variant, const GemmArgs &a, hipStream_t st);

}  // namespace zq
