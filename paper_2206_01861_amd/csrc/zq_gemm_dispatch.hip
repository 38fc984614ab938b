// Schedule selection for the GeMM calls (App. D: the schedule is chosen at run
// time from batch x sequence length so that padding is lowest; large token
// counts are ranked by matrix-core throughput, small ones by memory bandwidth).
#include "../../include/zq.h"
#include "zq_internal.h"

#include <mutex>
#include <vector>

namespace zq {

constexpr int kStreamMaxTokens = 128;   // the weight-streaming schedules hold up to eight 16-token tiles

hipError_t launch_gemm_simple(const GemmArgs &a, hipStream_t st);
hipError_t launch_gemm_tile(const GemmArgs &a, int block, hipStream_t st);
hipError_t launch_gemm_skinny(const GemmArgs &a, bool split_k, hipStream_t st);
size_t stream_workspace_bytes(int M, int N, int K, int w_bits);
void stream_plan(int M, int N, int K, int w_bits, bool allow_split, int *row_blocks, int *k_splits, int *consumers,
                 int *k_ranges);

// Measured overrides of the built-in choices (the profiler-driven schedule search of App. D, kept
// as a table the caller fills): exact (N, K, bits), a range of M.
namespace {
struct TuneEntry {
    int m_lo, m_hi, N, K, w_bits, variant, row_blocks, k_splits;
};
std::mutex g_tune_mutex;
std::vector<TuneEntry> g_tune;

bool tune_lookup(int M, int N, int K, int w_bits, TuneEntry *out) {
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    for (auto it = g_tune.rbegin(); it != g_tune.rend(); ++it) {     // the latest entry wins
        if (it->N == N && it->K == K && it->w_bits == w_bits && M >= it->m_lo && M <= it->m_hi) {
            *out = *it;
            return true;
        }
    }
    return false;
}
}  // namespace

bool tuned_stream_plan(int M, int N, int K, int w_bits, int *row_blocks, int *k_splits) {
    TuneEntry e;
    if (!tune_lookup(M, N, K, w_bits, &e) || e.row_blocks <= 0) return false;
    if (e.variant != kGemmSkinny && e.variant != kGemmSkinnySplitK) return false;
    *row_blocks = e.row_blocks;
    *k_splits = e.k_splits;
    return true;
}

size_t gemm_variant_workspace(int variant, int M, int N, int K, int w_bits) {
    if (variant == kGemmTileSplitK) return gemm_tile_split_workspace(M, N, K);
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
        case kGemmTile256x192:
            return true;                              // the last stage of a ragged K is zero filled
        case kGemmTileSplitK:
            return gemm_tile_splits(M, N, K) > 1 && workspace_bytes >= gemm_tile_split_workspace(M, N, K);
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
        case kGemmTile256x192: return launch_gemm_tile(a, 256192, st);
        case kGemmTileSplitK: return launch_gemm_tile_splitk(a, st);
        case kGemmSkinny: return launch_gemm_skinny(a, false, st);
        case kGemmSkinnySplitK: return launch_gemm_skinny(a, true, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace zq

extern "C" int zq_gemm_choose_variant(int M, int N, int K, int w_bits, size_t workspace_bytes) {
    using namespace zq;
    TuneEntry tuned;
    if (tune_lookup(M, N, K, w_bits, &tuned) &&
        gemm_variant_supports(tuned.variant, M, N, K, w_bits, workspace_bytes))
        return tuned.variant;
    // Up to 64 tokens every shape is bound by the weight stream; up to 128 tokens the streaming
    // schedules still win once K is long enough that the activation tile is a small part of the traffic.
    if (M <= 64 || (M <= kStreamMaxTokens && K >= 2048 && (K % 256) == 0)) {
        // 65 to 128 tokens against a long K and few tiles: the tiled K split is 5-12 % ahead of streaming
        if (M > 64 && gemm_variant_supports(kGemmTileSplitK, M, N, K, w_bits, workspace_bytes)) return kGemmTileSplitK;
        if (gemm_variant_supports(kGemmSkinnySplitK, M, N, K, w_bits, workspace_bytes) &&
            gemm_variant_workspace(kGemmSkinnySplitK, M, N, K, w_bits) > 0)
            return kGemmSkinnySplitK;
        if (gemm_variant_supports(kGemmSkinny, M, N, K, w_bits, 0)) return kGemmSkinny;
        // K not a multiple of 256: the tiled schedules below take it
    }
    // Tiny problems (a BERT-base layer at 128 tokens) are all latency: one wave per 16x16 tile straight
    // from global memory starts and finishes sooner than a handful of LDS-tiled workgroups (6.2 vs 6.8 us).
    if ((long)M * N * K <= (1L << 27)) return kGemmSimple;
    // Few tiles against a long K (some hundred tokens, a few thousand columns): split K over the idle
    // compute units when the caller's workspace holds the partial products.
    if (gemm_variant_supports(kGemmTileSplitK, M, N, K, w_bits, workspace_bytes)) return kGemmTileSplitK;
    // Tiled schedules.  The tiles of a launch all take the same time and a compute unit holds one of
    // them, so a launch lasts (rounds of tiles) x (time of a tile), and the time of a tile goes with
    // its area times a factor for the operand bytes it moves per product.  Factors fitted to one-round
    // measurements at K = 2048..6144 (256x256 = 1): 256x192 1.15, 128x128 1.85.
    constexpr long kComputeUnits = 256;
    const long rows256 = (M + 255) / 256;
    const long t256 = rows256 * ((N + 255) / 256);
    const long t192 = rows256 * ((N + 191) / 192);
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    auto rounds = [](long tiles, long slots) { return (tiles + slots - 1) / slots; };
    const long c256 = rounds(t256, kComputeUnits) * 65536 * 100;
    const long c192 = rounds(t192, kComputeUnits) * 49152 * 115;
    const long c128 = rounds(t128, kComputeUnits) * 16384 * 185;
    if (c128 <= c256 && c128 <= c192) return kGemmTile128;
    return (c192 < c256) ? kGemmTile256x192 : kGemmTile256;
}

extern "C" int zq_gemm_stream_plan(int M, int N, int K, int w_bits, size_t workspace_bytes, int *row_blocks,
                                   int *k_splits, int *consumers) {
    using namespace zq;
    if (row_blocks == nullptr || k_splits == nullptr || consumers == nullptr) return ZQ_ERR_NULL;
    if (M <= 0 || M > kStreamMaxTokens || N <= 0 || (N % 16) != 0 || K <= 0 || (K % 256) != 0 || (w_bits != 8 && w_bits != 4))
        return ZQ_ERR_UNSUPPORTED;
    const bool split = workspace_bytes > 0 && workspace_bytes >= stream_workspace_bytes(M, N, K, w_bits);
    int k_ranges = 1;
    stream_plan(M, N, K, w_bits, split, row_blocks, k_splits, consumers, &k_ranges);
    return ZQ_OK;
}

extern "C" int zq_gemm_stream_k_ranges(int M, int N, int K, int w_bits, size_t workspace_bytes) {
    using namespace zq;
    if (M <= 0 || M > kStreamMaxTokens || N <= 0 || (N % 16) != 0 || K <= 0 || (K % 256) != 0 || (w_bits != 8 && w_bits != 4))
        return 0;
    const bool split = workspace_bytes > 0 && workspace_bytes >= stream_workspace_bytes(M, N, K, w_bits);
    int row_blocks = 0, k_splits = 0, consumers = 0, k_ranges = 1;
    stream_plan(M, N, K, w_bits, split, &row_blocks, &k_splits, &consumers, &k_ranges);
    return k_ranges;
}

extern "C" int zq_tune_set(int m_lo, int m_hi, int N, int K, int w_bits, int variant, int row_blocks, int k_splits) {
    using namespace zq;
    if (m_lo <= 0 || m_hi < m_lo || N <= 0 || K <= 0 || (w_bits != 8 && w_bits != 4)) return ZQ_ERR_SHAPE;
    if (variant < 0 || variant >= kGemmVariantCount) return ZQ_ERR_UNSUPPORTED;
    const bool streaming = variant == kGemmSkinny || variant == kGemmSkinnySplitK;
    if (row_blocks != 0 || k_splits != 0) {
        if (!streaming || (N % 16) != 0 || (K % 256) != 0 || m_hi > kStreamMaxTokens) return ZQ_ERR_UNSUPPORTED;
        const int strips = N / 16, stages = K / 256;
        if (row_blocks < 1 || row_blocks > strips || (strips + row_blocks - 1) / row_blocks > 8) return ZQ_ERR_SHAPE;
        if (k_splits < 1 || k_splits > stages) return ZQ_ERR_SHAPE;
        if ((variant == kGemmSkinny) != (k_splits == 1)) return ZQ_ERR_SHAPE;   // a K split is the split schedule
        if (k_splits > 1 && (strips > 8192 || (double)k_splits * m_hi * N * 4.0 >= 2147483648.0)) return ZQ_ERR_SHAPE;
    }
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    g_tune.push_back(TuneEntry{m_lo, m_hi, N, K, w_bits, variant, row_blocks, k_splits});
    return ZQ_OK;
}

extern "C" void zq_tune_clear(void) {
    std::lock_guard<std::mutex> lock(zq::g_tune_mutex);
    zq::g_tune.clear();
}

extern "C" int zq_tune_count(void) {
    std::lock_guard<std::mutex> lock(zq::g_tune_mutex);
    return (int)zq::g_tune.size();
}
