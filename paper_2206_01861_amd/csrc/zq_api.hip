// C ABI of libzq: argument validation and dispatch.  Every check runs on the
// host before any HIP call, so a bad argument launches nothing.
#include "../../include/zq.h"
#include "zq_internal.h"

#include <atomic>

namespace {

std::atomic<int> g_forced_variant{-1};
std::atomic<int> g_in_kernel_quant{1};

inline bool is_tile_variant(int v) {
    return v == zq::kGemmTile128 || v == zq::kGemmTile256 || v == zq::kGemmTile256x128 ||
           v == zq::kGemmTile256x192;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

constexpr int kMaxRow = 32768;   // longest row the fused front-ends keep in registers
constexpr uint64_t kMaxOperandBytes = 1ull << 31;   // a GeMM operand must stay below 2 GiB
static_assert(ZQ_WORKSPACE_FIXED_BYTES == zq::kWsFixedBytes, "the header states the size of the fixed part");

zq_status check_rowquant(const void *in, const void *p0, const void *p1, int M, int K, const int8_t *xq,
                         const float *s_tok, const void *y_out, int y_dtype) {
    if (in == nullptr || xq == nullptr || s_tok == nullptr) return ZQ_ERR_NULL;
    if (M <= 0 || K <= 0 || (K % 16) != 0 || K > kMaxRow) return ZQ_ERR_SHAPE;
    if (y_dtype != 0 && y_dtype != 1) return ZQ_ERR_UNSUPPORTED;
    if (misaligned(in) || misaligned(p0) || misaligned(p1) || misaligned(xq) || misaligned(s_tok) ||
        misaligned(y_out))
        return ZQ_ERR_ALIGN;
    return ZQ_OK;
}

zq_status gemm_common(const int8_t *xq, const float *s_tok, const void *wq, const float *s_w, int groups,
                      const void *bias, int M, int N, int K, void *out, int32_t *acc_out, int8_t *out_q,
                      float *out_s_tok, void *workspace, size_t workspace_bytes, int w_bits, int act,
                      bool out_optional, zq_stream stream) {
    if (xq == nullptr || s_tok == nullptr || wq == nullptr || s_w == nullptr) return ZQ_ERR_NULL;
    if (out == nullptr && !(out_optional && out_q != nullptr)) return ZQ_ERR_NULL;
    if ((out_q == nullptr) != (out_s_tok == nullptr)) return ZQ_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || groups <= 0) return ZQ_ERR_SHAPE;
    if ((N % groups) != 0 || ((N / groups) % 16) != 0) return ZQ_ERR_SHAPE;
    if ((K % (w_bits == 4 ? 32 : 16)) != 0 || K > (w_bits == 4 ? ZQ_MAX_K_W4 : ZQ_MAX_K)) return ZQ_ERR_SHAPE;
    // the kernels address both operands through 32-bit buffer offsets
    if ((uint64_t)M * K >= kMaxOperandBytes || (uint64_t)N * K * w_bits / 8 >= kMaxOperandBytes) return ZQ_ERR_SHAPE;
    if (out_q != nullptr && N > kMaxRow) return ZQ_ERR_SHAPE;
    if (misaligned(xq) || misaligned(s_tok) || misaligned(wq) || misaligned(s_w) || misaligned(bias) ||
        misaligned(out) || misaligned(acc_out) || misaligned(out_q) || misaligned(out_s_tok) ||
        misaligned(workspace))
        return ZQ_ERR_ALIGN;
    if (workspace == nullptr) workspace_bytes = 0;

    int variant = g_forced_variant.load();
    if (variant >= 0) {
        if (!zq::gemm_variant_supports(variant, M, N, K, w_bits, workspace_bytes)) return ZQ_ERR_UNSUPPORTED;
    } else {
        variant = zq_gemm_choose_variant(M, N, K, w_bits, workspace_bytes);
    }
    // On the tiled schedules the output rows are quantized inside the GeMM kernel.
    const bool in_kernel = out_q != nullptr && g_in_kernel_quant.load() != 0 && is_tile_variant(variant) &&
                           zq::gemm_tile_quant_supported(M, N, workspace_bytes);
    if (out == nullptr && !in_kernel) return ZQ_ERR_UNSUPPORTED;
    zq::GemmArgs a;
    a.xq = xq; a.s_tok = s_tok; a.wq = wq; a.s_w = s_w; a.groups = groups; a.bias = bias;
    a.M = M; a.N = N; a.K = K; a.out = out; a.acc_out = acc_out;
    a.workspace = workspace; a.workspace_bytes = workspace_bytes; a.w_bits = w_bits; a.act = act;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (in_kernel) {
        a.q_out = out_q; a.q_scale_out = out_s_tok;
        return zq::launch_gemm_tile_quant(a, st) == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
    }
    if (zq::launch_gemm(variant, a, st) != hipSuccess) return ZQ_ERR_HIP;
    if (out_q != nullptr) {
        // Re-quantization for the next GeMM: token-wise quantizer over the FP16 row just written.
        if (zq::launch_rowquant(zq::kOpIdentity, out, nullptr, nullptr, 0.0f, M, N, out_q, out_s_tok, nullptr, 0,
                                st) != hipSuccess)
            return ZQ_ERR_HIP;
    }
    return ZQ_OK;
}

}  // namespace

extern "C" {

const char *zq_status_string(zq_status st) {
    switch (st) {
        case ZQ_OK: return "ok";
        case ZQ_ERR_NULL: return "a required pointer is NULL";
        case ZQ_ERR_SHAPE: return "bad shape: non-positive, not divisible as required, or too large";
        case ZQ_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case ZQ_ERR_UNSUPPORTED: return "unsupported bits, dtype, flag or forced schedule";
        case ZQ_ERR_HIP: return "the HIP runtime reported an error";
        case ZQ_ERR_SCRATCH: return "the shape needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

int zq_version(void) { return 100; }

zq_status zq_quantize_weight_groupwise(const void *w_fp16, int N, int K, int groups, int bits, void *wq_out,
                                       float *s_w_out, zq_stream stream) {
    if (w_fp16 == nullptr || wq_out == nullptr || s_w_out == nullptr) return ZQ_ERR_NULL;
    if (bits != 8 && bits != 4) return ZQ_ERR_UNSUPPORTED;
    if (N <= 0 || K <= 0 || groups <= 0 || groups > 65535) return ZQ_ERR_SHAPE;
    if ((N % groups) != 0 || ((N / groups) % 16) != 0) return ZQ_ERR_SHAPE;
    if ((K % (bits == 4 ? 32 : 16)) != 0) return ZQ_ERR_SHAPE;
    if (misaligned(w_fp16) || misaligned(wq_out) || misaligned(s_w_out)) return ZQ_ERR_ALIGN;
    hipError_t e = zq::launch_weight_quant(w_fp16, N, K, groups, bits, wq_out, s_w_out,
                                           reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

zq_status zq_layernorm_quant_tokenwise(const void *x_fp16, const void *gamma_fp16, const void *beta_fp16, float eps,
                                       int M, int K, int8_t *xq_out, float *s_tok_out, void *y_out, int y_dtype,
                                       zq_stream stream) {
    if (gamma_fp16 == nullptr) return ZQ_ERR_NULL;
    zq_status s = check_rowquant(x_fp16, gamma_fp16, beta_fp16, M, K, xq_out, s_tok_out, y_out, y_dtype);
    if (s != ZQ_OK) return s;
    if (!(eps >= 0.0f)) return ZQ_ERR_UNSUPPORTED;
    hipError_t e = zq::launch_rowquant(zq::kOpLayerNorm, x_fp16, gamma_fp16, beta_fp16, eps, M, K, xq_out, s_tok_out,
                                       y_out, y_dtype, reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

zq_status zq_gelu_quant_tokenwise(const void *h_fp16, const void *bias_fp16, int approx_tanh, int M, int N,
                                  int8_t *xq_out, float *s_tok_out, void *y_out, int y_dtype, zq_stream stream) {
    zq_status s = check_rowquant(h_fp16, bias_fp16, nullptr, M, N, xq_out, s_tok_out, y_out, y_dtype);
    if (s != ZQ_OK) return s;
    if (approx_tanh != 0 && approx_tanh != 1) return ZQ_ERR_UNSUPPORTED;
    hipError_t e = zq::launch_rowquant(approx_tanh ? zq::kOpGeluTanh : zq::kOpGeluErf, h_fp16, bias_fp16, nullptr,
                                       0.0f, M, N, xq_out, s_tok_out, y_out, y_dtype,
                                       reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

zq_status zq_quantize_tokenwise(const void *x_fp16, int M, int K, int8_t *xq_out, float *s_tok_out, zq_stream stream) {
    zq_status s = check_rowquant(x_fp16, nullptr, nullptr, M, K, xq_out, s_tok_out, nullptr, 0);
    if (s != ZQ_OK) return s;
    hipError_t e = zq::launch_rowquant(zq::kOpIdentity, x_fp16, nullptr, nullptr, 0.0f, M, K, xq_out, s_tok_out,
                                       nullptr, 0, reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

zq_status zq_dequantize_acc(const int32_t *acc, const float *s_tok, const float *s_w, int groups,
                            const void *bias_fp16, int M, int N, void *out_fp16, zq_stream stream) {
    if (acc == nullptr || s_tok == nullptr || s_w == nullptr || out_fp16 == nullptr) return ZQ_ERR_NULL;
    if (M <= 0 || N <= 0 || groups <= 0) return ZQ_ERR_SHAPE;
    if ((N % groups) != 0 || ((N / groups) % 16) != 0) return ZQ_ERR_SHAPE;
    if (misaligned(acc) || misaligned(s_tok) || misaligned(s_w) || misaligned(bias_fp16) || misaligned(out_fp16))
        return ZQ_ERR_ALIGN;
    hipError_t e = zq::launch_dequant(acc, s_tok, s_w, groups, bias_fp16, M, N, out_fp16,
                                      reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

size_t zq_gemm_workspace_bytes(int M, int N, int K, int w_bits) {
    if (M <= 0 || N <= 0 || K <= 0 || (w_bits != 8 && w_bits != 4)) return 0;
    size_t best = 0;
    for (int v = 0; v < zq::kGemmVariantCount; ++v) {
        size_t need = zq::gemm_variant_workspace(v, M, N, K, w_bits);
        if (need > best && zq::gemm_variant_supports(v, M, N, K, w_bits, need)) best = need;
    }
    return best;
}

size_t zq_gemm_quant_workspace_bytes(int M, int N, int K, int w_bits) {
    if (M <= 0 || N <= 0 || K <= 0 || (w_bits != 8 && w_bits != 4)) return 0;
    size_t need = zq_gemm_workspace_bytes(M, N, K, w_bits);
    // the schedule of a caller who offers exactly `need` (a larger offer changes nothing)
    const int variant = zq_gemm_choose_variant(M, N, K, w_bits, need);
    if (is_tile_variant(variant) && zq::gemm_tile_quant_supported(M, N, zq::kWsFixedBytes) && need < zq::kWsFixedBytes)
        need = zq::kWsFixedBytes;
    return need;
}

zq_status zq_workspace_init(void *workspace, size_t workspace_bytes, zq_stream stream) {
    if (workspace == nullptr) return ZQ_ERR_NULL;
    if (workspace_bytes < zq::kWsFixedBytes) return ZQ_ERR_SHAPE;
    if (misaligned(workspace)) return ZQ_ERR_ALIGN;
    return zq::launch_workspace_init(workspace, reinterpret_cast<hipStream_t>(stream)) == hipSuccess ? ZQ_OK
                                                                                                      : ZQ_ERR_HIP;
}

zq_status zq_gemm_i8_dequant(const int8_t *xq, const float *s_tok, const int8_t *wq, const float *s_w, int groups,
                             const void *bias_fp16, int M, int N, int K, void *out_fp16, int32_t *acc_out,
                             int8_t *out_q, float *out_s_tok, void *workspace, size_t workspace_bytes,
                             zq_stream stream) {
    return gemm_common(xq, s_tok, wq, s_w, groups, bias_fp16, M, N, K, out_fp16, acc_out, out_q, out_s_tok,
                       workspace, workspace_bytes, 8, 0, false, stream);
}

zq_status zq_gemm_w4a8_dequant(const int8_t *xq, const float *s_tok, const uint8_t *wq4, const float *s_w,
                               int groups, const void *bias_fp16, int M, int N, int K, void *out_fp16,
                               int32_t *acc_out, int8_t *out_q, float *out_s_tok, void *workspace,
                               size_t workspace_bytes, zq_stream stream) {
    return gemm_common(xq, s_tok, wq4, s_w, groups, bias_fp16, M, N, K, out_fp16, acc_out, out_q, out_s_tok,
                       workspace, workspace_bytes, 4, 0, false, stream);
}

zq_status zq_gemm_gelu_quant_tokenwise(const int8_t *xq, const float *s_tok, const void *wq, int w_bits,
                                       const float *s_w, int groups, const void *bias_fp16, int approx_tanh, int M,
                                       int N, int K, void *g_fp16, int8_t *gq_out, float *s_tok_out,
                                       void *workspace, size_t workspace_bytes, zq_stream stream) {
    if (w_bits != 8 && w_bits != 4) return ZQ_ERR_UNSUPPORTED;
    if (approx_tanh != 0 && approx_tanh != 1) return ZQ_ERR_UNSUPPORTED;
    if (gq_out == nullptr || s_tok_out == nullptr) return ZQ_ERR_NULL;
    return gemm_common(xq, s_tok, wq, s_w, groups, bias_fp16, M, N, K, g_fp16, nullptr, gq_out, s_tok_out, workspace,
                       workspace_bytes, w_bits, approx_tanh ? 2 : 1, true, stream);
}

namespace {
constexpr int kA16StreamTokens = 128;   // FP16 activations: weight streaming up to here, in launches of 64 tokens
}

// 65 to 128 tokens: the tiled schedule with a K split where it divides K at least three ways (measured
// ahead of two streaming launches there: 4096x4096 at 128 tokens 32.5 -> 21 us), else streaming.
static bool a16_tiles_with_split(int M, int N, int K) {
    if (M <= 64) return false;
    const int ks = zq::gemm_a16_tile_splits(M, N, K);
    return ks >= ((M <= kA16StreamTokens && (K % 256) == 0) ? 3 : 2);
}

size_t zq_gemm_w8a16_workspace_bytes(int M, int N, int K) {
    if (M <= 0 || N <= 0 || K <= 0 || (N % 16) != 0 || (K % 16) != 0) return 0;
    size_t need = 0;
    if (M <= kA16StreamTokens && (K % 256) == 0) need = zq::stream_a16_workspace_bytes(M < 64 ? M : 64, N, K);
    if (a16_tiles_with_split(M, N, K)) {
        const size_t t = zq::gemm_a16_tile_split_workspace(M, N, K);
        if (t > need) need = t;
    }
    return need;
}

int zq_gemm_w8a16_stream_plan(int M, int N, int K, size_t workspace_bytes, int *row_blocks, int *k_splits,
                              int *consumers) {
    if (row_blocks == nullptr || k_splits == nullptr || consumers == nullptr) return ZQ_ERR_NULL;
    if (M <= 0 || M > 64 || N <= 0 || (N % 16) != 0 || K <= 0 || (K % 256) != 0) return ZQ_ERR_UNSUPPORTED;
    const size_t need = zq::stream_a16_workspace_bytes(M, N, K);
    zq::stream_a16_plan(M, N, K, need > 0 && workspace_bytes >= need, row_blocks, k_splits, consumers);
    return ZQ_OK;
}

zq_status zq_gemm_w8a16_dequant(const void *x_fp16, const int8_t *wq, const float *s_w, int groups,
                                const void *bias_fp16, int M, int N, int K, void *out_fp16, void *workspace,
                                size_t workspace_bytes, zq_stream stream) {
    if (x_fp16 == nullptr || wq == nullptr || s_w == nullptr || out_fp16 == nullptr) return ZQ_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || groups <= 0) return ZQ_ERR_SHAPE;
    if ((N % groups) != 0 || ((N / groups) % 16) != 0) return ZQ_ERR_SHAPE;
    if ((K % 16) != 0 || K > ZQ_MAX_K) return ZQ_ERR_SHAPE;
    if ((uint64_t)M * K * 2 >= kMaxOperandBytes || (uint64_t)N * K >= kMaxOperandBytes) return ZQ_ERR_SHAPE;
    if (misaligned(x_fp16) || misaligned(wq) || misaligned(s_w) || misaligned(bias_fp16) || misaligned(out_fp16) ||
        misaligned(workspace))
        return ZQ_ERR_ALIGN;
    if (workspace == nullptr) workspace_bytes = 0;
    zq::A16Args a;
    a.x = x_fp16; a.wq = wq; a.s_w = s_w; a.groups = groups; a.bias = bias_fp16;
    a.M = M; a.N = N; a.K = K; a.out = out_fp16; a.workspace = workspace; a.workspace_bytes = workspace_bytes;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    hipError_t e;
    const bool tile_split = a16_tiles_with_split(M, N, K) &&
                            workspace_bytes >= zq::gemm_a16_tile_split_workspace(M, N, K);
    if (tile_split) {
        e = zq::launch_gemm_a16_tile(a, st);
    } else if (M <= kA16StreamTokens && (K % 256) == 0) {
        // Weight streaming holds up to 64 tokens per launch; 65..128 tokens run as two launches over
        // row halves (the weights are read twice, which is still well ahead of the tiled schedule on
        // so few rows).  The K split is taken only when the workspace holds its fp32 partials.
        e = hipSuccess;
        for (int m0 = 0; m0 < M && e == hipSuccess; m0 += 64) {
            zq::A16Args h = a;
            h.M = (M - m0) < 64 ? (M - m0) : 64;
            h.x = static_cast<const uint16_t *>(x_fp16) + (size_t)m0 * K;
            h.out = static_cast<uint16_t *>(out_fp16) + (size_t)m0 * N;
            const size_t need = zq::stream_a16_workspace_bytes(h.M, N, K);
            e = zq::launch_gemm_a16_stream(h, need > 0 && workspace_bytes >= need, st);
        }
    } else if ((long)M * N * K > (1L << 27)) {
        e = zq::launch_gemm_a16_tile(a, st);
    } else {
        e = zq::launch_gemm_a16_simple(a, st);
    }
    return e == hipSuccess ? ZQ_OK : ZQ_ERR_HIP;
}

}  // extern "C"

// The workspace of zq_gemm_i8_dequant_static: one array per device, part of the loaded code
// object (zero when the library is loaded, which is the state zq_workspace_init establishes).
// In host code the name `scratch` only stands for the symbol; its address on a device comes from
// hipGetSymbolAddress, asked once per device with that device current.
namespace {
constexpr size_t kScratchBytes = ZQ_STATIC_SCRATCH_BYTES;
static_assert(kScratchBytes > zq::kWsFixedBytes && kScratchBytes % 256 == 0, "fixed part plus room for partial sums");
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
std::atomic<void *> g_scratch_ptr[64];

hipError_t scratch_on_current_device(void **out) {
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread gets the same answer
    }
    *out = p;
    return hipSuccess;
}
}  // namespace

extern "C" {

zq_status zq_gemm_i8_dequant_static(const int8_t *xq, const float *s_tok, const int8_t *wq, const float *s_w,
                                    int groups, const void *bias_fp16, int M, int N, int K, void *out_fp16,
                                    int32_t *acc_out, int8_t *out_q, float *out_s_tok, zq_stream stream) {
    // Shape errors first, as in the plain call; then the size of the scratch this shape would use.
    if (M > 0 && N > 0 && K > 0) {
        const size_t need = out_q != nullptr ? zq_gemm_quant_workspace_bytes(M, N, K, 8)
                                             : zq_gemm_workspace_bytes(M, N, K, 8);
        if (need > kScratchBytes) return ZQ_ERR_SCRATCH;
    }
    if (xq == nullptr || s_tok == nullptr || wq == nullptr || s_w == nullptr || out_fp16 == nullptr)
        return ZQ_ERR_NULL;
    void *ws = nullptr;
    if (scratch_on_current_device(&ws) != hipSuccess) return ZQ_ERR_HIP;
    return gemm_common(xq, s_tok, wq, s_w, groups, bias_fp16, M, N, K, out_fp16, acc_out, out_q, out_s_tok, ws,
                       kScratchBytes, 8, 0, false, stream);
}

int zq_debug_force_gemm_variant(int variant) {
    if (variant >= zq::kGemmVariantCount) variant = -1;
    return g_forced_variant.exchange(variant < 0 ? -1 : variant);
}

int zq_debug_set_in_kernel_quant(int on) { return g_in_kernel_quant.exchange(on != 0 ? 1 : 0); }

int zq_gemm_quantizes_in_kernel(int M, int N, int K, int w_bits, size_t workspace_bytes) {
    if (M <= 0 || N <= 0 || K <= 0 || (w_bits != 8 && w_bits != 4)) return 0;
    int variant = g_forced_variant.load();
    if (variant < 0) variant = zq_gemm_choose_variant(M, N, K, w_bits, workspace_bytes);
    return (g_in_kernel_quant.load() != 0 && is_tile_variant(variant) &&
            zq::gemm_tile_quant_supported(M, N, workspace_bytes))
               ? 1
               : 0;
}

zq_status zq_quant_wait_expired(void *workspace, int *count_out) {
    if (workspace == nullptr || count_out == nullptr) return ZQ_ERR_NULL;
    if (misaligned(workspace)) return ZQ_ERR_ALIGN;
    unsigned *word = zq::ws_control(workspace) + 2;
    unsigned c = 0, zero = 0;
    if (hipMemcpy(&c, word, sizeof(unsigned), hipMemcpyDeviceToHost) != hipSuccess) return ZQ_ERR_HIP;
    if (hipMemcpy(word, &zero, sizeof(unsigned), hipMemcpyHostToDevice) != hipSuccess) return ZQ_ERR_HIP;
    *count_out = (int)c;
    return ZQ_OK;
}

const char *zq_gemm_variant_name(int variant) {
    switch (variant) {
        case zq::kGemmSimple: return "simple";
        case zq::kGemmTile128: return "tile128";
        case zq::kGemmTile256: return "tile256";
        case zq::kGemmSkinny: return "skinny";
        case zq::kGemmSkinnySplitK: return "skinny_splitk";
        case zq::kGemmTile256x128: return "tile256x128";
        case zq::kGemmTile256x192: return "tile256x192";
        case zq::kGemmTileSplitK: return "tile128_splitk";
    }
    return nullptr;
}

}  // extern "C"
