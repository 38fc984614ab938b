// Schedule selection for the GeMM calls (App. D: the schedule is chosen at run
// time from batch x sequence length so that padding is lowest; large token
// counts are ranked by matrix-core throughput, small ones by memory bandwidth).
#include "../../include/zq.h"
#include "zq_internal.h"

namespace zq {

constexpr int kStreamMaxTokens = 128;   // the weight-streaming schedules hold up to eight 16-token tiles

hipError_t launch_gemm_simple(const GemmArgs &a, hipStream_t st);
hipError_t launch_gemm_tile(const GemmArgs &a, int block, hipStream_t st);
hipError_t launch_gemm_skinny(const GemmArgs &a, bool split_k, hipStream_t st);
size_t stream_workspace_bytes(int M, int N, int K, int w_bits);
void stream_plan(int M, int N, int K, int w_bits, bool allow_split, int *row_blocks, int *k_splits, int *consumers);

size_t gemm_variant_workspace(int variant, int M, int N, int K, int w_bits) {
    if (variant != kGemmSkinnySplitK || M > kStreamMaxTokens || (K % 256) != 0) return 0;
    return stream_workspace_bytes(M, N, K, w_bits);
}

bool gemm_variant_supports(int variant, int M, int N, int K, int w_bits, size_t workspace_bytes) {
    switch (variant) {
        case kGemmSimple:
            return true;
        case kGemmTile128:
        case kGemmTile256:
        case kGemmTile256x128:
            return (K % 128) == 0;
        case kGemmSkinny:
            return M <= kStreamMaxTokens && (K % 256) == 0;
        case kGemmSkinnySplitK:
            return M <= kStreamMaxTokens && (K % 256) == 0 &&
                   workspace_bytes >= gemm_variant_workspace(variant, M, N, K, w_bits);
    }
    return false;
}

hipError_t launch_gemm(int variant, const GemmArgs &a, hipStream_t st) {
    switch (variant) {
        case kGemmSimple: return launch_gemm_simple(a, st);
        case kGemmTile128: return launch_gemm_tile(a, 128, st);
        case kGemmTile256: return launch_gemm_tile(a, 256, st);
        case kGemmTile256x128: return launch_gemm_tile(a, 192, st);
        case kGemmSkinny: return launch_gemm_skinny(a, false, st);
        case kGemmSkinnySplitK: return launch_gemm_skinny(a, true, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace zq

extern "C" int zq_gemm_choose_variant(int M, int N, int K, int w_bits, size_t workspace_bytes) {
    using namespace zq;
    // Up to 64 tokens every shape is bound by the weight stream; up to 128 tokens the streaming
    // schedules still win once K is long enough that the activation tile is a small part of the traffic.
    if (M <= 64 || (M <= kStreamMaxTokens && K >= 2048 && (K % 256) == 0)) {
        if (gemm_variant_supports(kGemmSkinnySplitK, M, N, K, w_bits, workspace_bytes) &&
            gemm_variant_workspace(kGemmSkinnySplitK, M, N, K, w_bits) > 0)
            return kGemmSkinnySplitK;
        if (gemm_variant_supports(kGemmSkinny, M, N, K, w_bits, 0)) return kGemmSkinny;
        if (M <= 64) return kGemmSimple;
    }
    if ((K % 128) != 0) return kGemmSimple;
    // 256x256 tiles once they fill the chip; 128x128 tiles waste less on ragged or small problems.
    const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256);
    if (t256 >= 160) return kGemmTile256;
    return kGemmTile128;
}

extern "C" int zq_gemm_stream_plan(int M, int N, int K, int w_bits, size_t workspace_bytes, int *row_blocks,
                                   int *k_splits, int *consumers) {
    using namespace zq;
    if (row_blocks == nullptr || k_splits == nullptr || consumers == nullptr) return ZQ_ERR_NULL;
    if (M <= 0 || M > kStreamMaxTokens || N <= 0 || (N % 16) != 0 || K <= 0 || (K % 256) != 0 || (w_bits != 8 && w_bits != 4))
        return ZQ_ERR_UNSUPPORTED;
    const bool split = workspace_bytes > 0 && workspace_bytes >= stream_workspace_bytes(M, N, K, w_bits);
    stream_plan(M, N, K, w_bits, split, row_blocks, k_splits, consumers);
    return ZQ_OK;
}
