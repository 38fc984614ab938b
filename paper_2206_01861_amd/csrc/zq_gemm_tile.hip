// LDS-tiled INT8 GeMM with the dequantization epilogue for large token counts
// (Sec. 4.3 "INT8 GeMM"; App. D "Dequantization Associated with GeMM
// Schedule").  Bound by the INT8 matrix cores.
//
// A workgroup of WAVES_M x WAVES_N waves owns a BM x BN output tile.  Per BK
// bytes of K both operand tiles go from global memory straight into LDS with
// 16-byte direct loads (no register staging) through a ring of NSTAGE stages;
// rows are BK bytes with their 16-byte chunks XOR-swizzled so that the
// ds_read_b128 of a matrix-core fragment (32 rows, one chunk) is free of bank
// conflicts.  Each wave computes (BN/WAVES_N) x (BM/WAVES_M) with
// v_mfma_i32_32x32x32_i8, the weight fragment as the first operand, so every
// group of four accumulator registers runs along the output columns.  Two
// fragment sets alternate so the LDS reads of k step s+1 are in flight under
// the MFMAs of step s; with two waves per SIMD the barrier and epilogue of one
// wave overlap the matrix-core work of the other.
//
// The epilogue scales the INT32 accumulators by s_tok[row] * s_w[group], adds
// the bias and rounds to FP16 (scales and bias were staged in LDS under the
// first operand loads), passes 32 rows at a time through a wave-private LDS
// buffer and writes full contiguous row segments.  INT4 weights are unpacked
// to INT8 (times 16) on their way into LDS and the factor is shifted out of
// the accumulator.
//
// QOUT = 1 adds the token-wise quantization of the output rows (App. A.2) to
// the epilogue: the tiles of a band of token rows exchange their row maxima
// through device memory and write INT8 codes from the accumulator registers
// (see the state block below and the end of the kernel).
//
// KSPLIT = 1 serves shapes with so few tiles that most compute units would
// idle while each tile walks a long K: several workgroups share a tile, each
// over its own range of K stages, and write raw accumulators to a workspace;
// splitk_finish_kernel adds them and applies the epilogue.
//
// KT = 2 (128 x 128 tile, INT8 weights) splits the eight waves into two teams
// that share every stage and take half of its k steps each, so that a wave
// owns 64 x 64 instead of 64 x 32; the teams add their accumulators through
// LDS after the last stage.
//
// XT = 1, 2 is the product of FP16 activations with INT8 weights (Sec. 5, the
// W8A16 setting): FP16 matrix-core instructions, fp32 accumulators, the
// weights made FP16 exactly either after the fragment read (XT = 1: INT8 in
// LDS) or on their way into LDS (XT = 2).  XT = 3 is XT = 1's operand path
// for INT4 weights under INT8 activations: the nibbles stay packed in LDS
// (direct loads, half the bytes) and are unpacked after the fragment read.
//
// Workgroup ids are remapped so that the workgroups an XCD receives
// (round-robin by id) cover a compact block of tiles and share operand panels
// in that XCD's L2.
#include <type_traits>

#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

namespace {

constexpr uint32_t kRsrcFlags = 0x00020000u;
typedef __attribute__((address_space(3))) void lds_void;

// Chunk swizzle: 16 consecutive rows reading the same logical chunk hit 16 different bank groups.
template <int BK>
__device__ __forceinline__ int swz(int row) {
    return (BK == 128) ? ((row & 7) ^ ((row >> 3) & 1)) : ((row >> 2) & 3);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// Eight nibbles -> two words of int8 (value x16) in natural k order.
__device__ __forceinline__ void unpack8_nat(uint32_t p, uint32_t &d0, uint32_t &d1) {
    const uint32_t lo = (p << 4) & 0xf0f0f0f0u;   // k 0,2,4,6
    const uint32_t hi = p & 0xf0f0f0f0u;          // k 1,3,5,7
    d0 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);   // lo0 hi0 lo1 hi1
    d1 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);   // lo2 hi2 lo3 hi3
}

// In-kernel output quantization (QOUT = 1).  The tiles that share a band of token rows publish
// the row maxima of their tile in the exchange slots of the caller's workspace, one 8-byte slot per
// (tile, row): the float bits of max |g| below, a tag above.  The tag is the workspace's launch
// generation plus one, so a slot counts only if the running launch wrote it and nothing is ever
// cleared; the last workgroup of a launch to finish reading moves the generation on (the device does
// it, so replaying a captured launch works).  The state lives in the workspace: calls on different
// workspaces are independent, calls sharing one must be ordered on a stream.
constexpr unsigned kQuantSpinLimit = 1u << 20;        // polls of ~1 us: about a second, far beyond any launch
constexpr unsigned kPoisonBits = 0x7fc00000u;         // a NaN; as an integer it is above the bits of every finite |g|

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NSTAGE, int KT = 1, int XT = 0>
struct TileCfg {
    static constexpr int kWaves = WAVES_M * WAVES_N * KT;
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kStage = BM * BK + BN * ((XT == 1 || XT == 3) ? BK / 2 : BK);   // XT = 1, 3: weight rows half as long as activation rows
    static constexpr int kWN = BN / WAVES_N;
    static constexpr int kEpiRow = kWN * 2 + 16;              // padded FP16 row of the wave-private buffer
    static constexpr int kEpi = kWaves * 32 * kEpiRow;
    static constexpr int kMain = NSTAGE * kStage > kEpi ? NSTAGE * kStage : kEpi;
    static constexpr int kLds = kMain + (2 * BN + BM) * 4;    // + column scale, column bias, row scale
    static constexpr int kLdsQ = kLds + (WAVES_N + 1) * BM * 4;   // + per-wave row maxima, row 1/scale
    static constexpr int kXchg = (kEpi + 15) / 16 * 16;       // K teams: where the accumulator exchange starts
    static_assert(BM * BN <= kMain, "the INT8 code tile reuses the stage ring");
    static_assert(KT == 1 || kXchg + BM * BN * 4 / 2 * KT <= NSTAGE * kStage, "the accumulator exchange reuses the stage ring");
};

}  // namespace


// KSPLIT = 1: the launch holds k_splits workgroups per tile, each multiplies its own range of K stages
// and writes the raw accumulators of its tile to partial[split][M][N] (INT32, or fp32 bits with
// XT = 1); a second kernel adds the splits and applies the epilogue (splitk_finish_kernel below).
//
// KT = 2: two teams of WAVES_M x WAVES_N waves share the tile and every stage in LDS; team t multiplies
// k steps t*KSTEPS/2 .. of each stage, so a wave owns a tile twice as large as it would with all waves
// side by side (a third fewer fragment reads per matrix-core instruction, and twice as many
// instructions between a fragment read and its use).  After the last stage the teams exchange half of
// their accumulators through LDS and each finishes half of the rows.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NSTAGE, int WBITS, int XT = 0, int QOUT = 0,
          int KSPLIT = 0, int KT = 1>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * KT, (WAVES_M * WAVES_N * KT >= 8) ? 1 : 2) void gemm_tile_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ s_tok, const uint8_t *__restrict__ wq,
    const float *__restrict__ s_w, int gs, const half_t *__restrict__ bias, int M, int N, int K,
    half_t *__restrict__ out, int32_t *__restrict__ acc_out, int tiles_m, int tiles_n, int act,
    int8_t *__restrict__ q_out, float *__restrict__ q_scale_out, int k_splits, int32_t *__restrict__ partial,
    unsigned long long *__restrict__ q_slots, unsigned *__restrict__ q_ctl) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
    using Cfg = TileCfg<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, KT, XT>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int NW = Cfg::kWaves;
    constexpr int NT = Cfg::kThreads;
    constexpr int X_STAGE = BM * BK;
    constexpr int STAGE = Cfg::kStage;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int KSTEPS = BK / 32;
    constexpr int KS_T = KSTEPS / KT;                // k steps of a stage that one team multiplies
    static_assert(KT == 1 || KT == 2, "one or two K teams");
    static_assert(KT == 1 || (QOUT == 0 && KSPLIT == 0), "K teams go with the plain epilogue");
    static_assert(KT == 1 || FM % KT == 0, "each team finishes a whole number of 32-row blocks");
    constexpr int CPR = BK / 16;                     // 16-byte chunks per row
    constexpr int RPU = 64 / CPR;                    // rows per 1 KB load unit
    constexpr int XU = BM / RPU;                     // load units in the activation tile
    // XT = 1, 2: FP16 activations (W8A16); the MFMA is the FP16 one and an activation row of a stage is still
    // BK bytes, now BK/2 values of K.
    // XT = 1: the weight rows stay INT8 in LDS (BK/2 bytes per stage, direct loads like the activations) and
    // become FP16 in registers after the fragment read: one 16-byte read holds the weights of two k
    // steps, converted exactly by cvt8_i8_f16.  So that a lane's sixteen weights meet the right
    // activations, the k steps of a stage take the activation chunks in a permuted order (see
    // read_x_paired): a sum over K does not depend on the order of K.
    // XT = 2: the weights take the register path of the INT4 weights (16 source bytes -> two 16-byte
    // chunks) with the same conversion instead of the nibble unpack, and sit in LDS as FP16.
    // XT = 3: INT8 activations, INT4 weights packed in LDS (again BK/2 bytes of a weight row per stage):
    // XT = 1's loop with the nibble unpack as the conversion and the INT8 MFMA.
    constexpr bool A16 = XT == 1 || XT == 2;
    constexpr bool PAIRED = XT == 1 || XT == 3;      // weight rows half as long as activation rows, widened after the fragment read
    constexpr int BKW = PAIRED ? BK / 2 : BK;        // bytes of a weight row per stage
    constexpr int CPRW = BKW / 16;
    constexpr int RPUW = 64 / CPRW;
    constexpr int WU = BN / RPUW;
    constexpr bool STAGED_W = (WBITS == 4 && XT != 3) || (XT == 2);   // weights that pass through registers on their way into LDS
    constexpr int XB = A16 ? 2 : 1;                  // bytes per activation value
    static_assert(!A16 || WBITS == 8, "FP16 activations go with INT8 weights");
    static_assert(XT != 3 || WBITS == 4, "packed weight rows in LDS are the INT4 ones");
    static_assert(!PAIRED || (BK == 128 && KT == 1), "the paired loop is written for four k steps per stage");
    static_assert(QOUT == 0 || XT == 0, "the output quantization is built for the INT8 product");
    static_assert(KSPLIT == 0 || QOUT == 0, "a K split leaves the epilogue to the second kernel");
    static_assert(XU % NW == 0, "activation load units must split evenly over the waves");
    constexpr int LX = XU / NW;                      // activation loads per wave per stage
    // weight loads per wave per stage; where the units do not split evenly some waves load a unit a
    // second time (the same bytes to the same place), so that every wave issues the same number of loads
    constexpr int LWD = STAGED_W ? 0 : (WU + NW - 1) / NW;
    using AccT = typename std::conditional<A16, float32x16, int32x16>::type;
    constexpr int LPS = LX + LWD;                    // direct loads per wave per stage
    constexpr int TPR4 = BK / 32;                    // INT4: threads per row (16 packed bytes each)
    constexpr int W4_ROWS = NT / TPR4;               // rows per pass
    constexpr int W4_PASSES = (BN + W4_ROWS - 1) / W4_ROWS;

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);

    // ---- tile coordinates, XCD aware --------------------------------------
    // QOUT: the tiles of one band of token rows have consecutive ids.  A tile waits for the others of
    // its band in the epilogue, and workgroups start in id order on every XCD, so the oldest
    // unfinished band always has all its tiles running.  (Round-robin over the XCDs still gives each
    // XCD a fixed set of weight column tiles.)
    int tm, tn;
    int split = 0;                                   // KSPLIT: which range of K stages this workgroup takes
    if constexpr (KSPLIT == 1) {
        split = blockIdx.x % k_splits;               // the splits of a tile have consecutive ids
        const int t = blockIdx.x / k_splits;
        tm = t / tiles_n;
        tn = t % tiles_n;
    } else if constexpr (QOUT == 1) {
        tm = blockIdx.x / tiles_n;
        tn = blockIdx.x % tiles_n;
    } else {
        const int nb = tiles_m * tiles_n;
        const int b = blockIdx.x;
        const int xcd = b % 8;
        const int per = nb / 8, rem = nb % 8;
        const int t = xcd * per + (xcd < rem ? xcd : rem) + b / 8;   // XCD x owns a contiguous run of logical tiles
        constexpr int GM = 8;                                        // tile rows per band
        const int band = t / (GM * tiles_n);
        const int band_rows = (tiles_m - band * GM) < GM ? (tiles_m - band * GM) : GM;
        const int within = t - band * GM * tiles_n;
        tm = band * GM + within % band_rows;
        tn = within / band_rows;
    }
    const int m0 = tm * BM;
    const int n0 = tn * BN;

    const int wrow_bytes = (WBITS == 8) ? K : K / 2;
    const int xrow_bytes = K * XB;
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(wq), 0, (int)((size_t)N * wrow_bytes), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(xq), 0, (int)((size_t)M * xrow_bytes), kRsrcFlags);

    // ---- per-lane source offsets of this wave's direct-load units ---------
    // Wave w takes units w, w+NW, ...; units below XU are activation rows, the
    // rest weight rows.  Rows past the matrix edge are clamped to the last row:
    // loaded, multiplied, never stored.
    int voff[LPS];
    // weight unit of this wave's load i (wave-uniform; a subtraction, not a remainder, which would go
    // through the vector unit and make the LDS address of the load look divergent)
    static_assert(LWD * NW <= 2 * WU || STAGED_W, "a unit is loaded at most twice");
    auto w_unit = [&](int i) {
        const int u = wave + NW * (i - LX);
        return __builtin_amdgcn_readfirstlane(u >= WU ? u - WU : u);
    };
#pragma unroll
    for (int i = 0; i < LPS; ++i) {
        if (i < LX) {
            const int row = (wave + NW * i) * RPU + lane / CPR;
            int grow = m0 + row;
            if (grow > M - 1) grow = M - 1;
            voff[i] = grow * xrow_bytes + (((lane % CPR) ^ swz<BK>(row)) * 16);
        } else {
            const int row = w_unit(i) * RPUW + lane / CPRW;
            int grow = n0 + row;
            if (grow > N - 1) grow = N - 1;
            voff[i] = grow * wrow_bytes + (((lane % CPRW) ^ swz<BKW>(row)) * 16);
        }
    }
    // K need not be a multiple of the stage depth: in the last stage the chunks past the end of a
    // row are fetched from an offset beyond the buffer, which the hardware answers with zeros (a
    // plain offset would run into the next row); zero operands add nothing to the product.
    constexpr int kNowhere = 0x7ffffff0;
    const int tail_bytes = xrow_bytes % BK;           // valid bytes of the last stage row, 0 = full
    const int tail_bytes_w = tail_bytes / (PAIRED ? 2 : XB);   // the same values of K in a weight row
    int voff_tail[LPS];
#pragma unroll
    for (int i = 0; i < LPS; ++i) {
        if (i < LX) {
            const int row = (wave + NW * i) * RPU + lane / CPR;
            const int chunk = (lane % CPR) ^ swz<BK>(row);
            voff_tail[i] = (tail_bytes == 0 || chunk * 16 < tail_bytes) ? voff[i] : kNowhere;
        } else {
            const int row = w_unit(i) * RPUW + lane / CPRW;
            const int chunk = (lane % CPRW) ^ swz<BKW>(row);
            voff_tail[i] = (tail_bytes == 0 || chunk * 16 < tail_bytes_w) ? voff[i] : kNowhere;
        }
    }
    // INT4 weights: thread -> (row = pass*W4_ROWS + tid/TPR4, 16 packed bytes = 32 codes = chunks 2q, 2q+1)
    int w4_voff[W4_PASSES];
    if (STAGED_W) {
#pragma unroll
        for (int p = 0; p < W4_PASSES; ++p) {
            int grow = n0 + p * W4_ROWS + (int)threadIdx.x / TPR4;
            if (grow > N - 1) grow = N - 1;
            w4_voff[p] = grow * wrow_bytes + ((int)threadIdx.x % TPR4) * 16;
        }
    }

    const int nkt = (xrow_bytes + BK - 1) / BK;
    // stages kt0 .. kt0 + n_loc - 1 are this workgroup's; all of them without a K split
    int kt0 = 0, n_loc = nkt;
    if constexpr (KSPLIT == 1) {
        const int base = nkt / k_splits, rem = nkt % k_splits;   // the launcher keeps k_splits <= nkt
        kt0 = split * base + (split < rem ? split : rem);
        n_loc = base + (split < rem ? 1 : 0);
    }
    // `beyond`: the stage lies past this workgroup's range of K.  The loads are issued all the same,
    // from an offset outside the buffer (the hardware writes zeros into the slot, which is free):
    // with the same number of loads at every stage boundary the wait counts are constants and the
    // boundary needs no branch, so the compiler can interleave the fragment reads that follow it
    // with the matrix-core instructions of the stage's last k step.  (Whether it then selects the
    // offsets or still branches around the loads varies between instantiations; forcing the
    // selection with masks it cannot see through measured level on INT8 and 2-3 % slower on INT4
    // weights and FP16 activations, so the expressions are left as they read best.)
    auto issue_direct = [&](int kt, int slot, bool beyond) {
        uint8_t *base = smem + slot * STAGE;
        const bool last = kt == nkt - 1;
        // the stage's byte offset inside a row is the same for every lane: said explicitly, so that it is
        // never taken for a per-lane value (which would wrap each load in a loop over its distinct values)
        const int so_x = __builtin_amdgcn_readfirstlane(beyond ? 0 : kt * BK);
        const int so_w = __builtin_amdgcn_readfirstlane(beyond ? 0 : kt * BKW);
#pragma unroll
        for (int i = 0; i < LPS; ++i) {
            const int vo = beyond ? kNowhere : (last ? voff_tail[i] : voff[i]);
            if (i < LX)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(base + (wave + NW * i) * 1024), 16, vo, so_x,
                                                         0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, (lds_void *)(base + X_STAGE + w_unit(i) * 1024), 16, vo,
                                                         so_w, 0, 0);
        }
    };
    int32x4 w4_regs[W4_PASSES];
    auto w4_fetch = [&](int kt, bool beyond) {
#pragma unroll
        for (int p = 0; p < W4_PASSES; ++p) {
            const bool inside = !beyond && kt * (BK / 2) + ((int)threadIdx.x % TPR4) * 16 < wrow_bytes;
            w4_regs[p] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, inside ? w4_voff[p] : kNowhere,
                                                               beyond ? 0 : kt * (BK / 2), 0);
        }
    };
    auto w4_store = [&](int slot) {
        uint8_t *base = smem + slot * STAGE + X_STAGE;
#pragma unroll
        for (int p = 0; p < W4_PASSES; ++p) {
            const int row = p * W4_ROWS + (int)threadIdx.x / TPR4;
            const int q = (int)threadIdx.x % TPR4;
            if (BN % W4_ROWS == 0 || row < BN) {   // the last pass may reach past the tile
                uint32_t d[8];
                if (XT == 2) {
                    const uint32x4_t lo = __builtin_bit_cast(
                        uint32x4_t, cvt8_i8_f16((uint32_t)w4_regs[p][0], (uint32_t)w4_regs[p][1]));
                    const uint32x4_t hi = __builtin_bit_cast(
                        uint32x4_t, cvt8_i8_f16((uint32_t)w4_regs[p][2], (uint32_t)w4_regs[p][3]));
                    d[0] = lo[0]; d[1] = lo[1]; d[2] = lo[2]; d[3] = lo[3];
                    d[4] = hi[0]; d[5] = hi[1]; d[6] = hi[2]; d[7] = hi[3];
                } else {
                    unpack8_nat((uint32_t)w4_regs[p][0], d[0], d[1]);
                    unpack8_nat((uint32_t)w4_regs[p][1], d[2], d[3]);
                    unpack8_nat((uint32_t)w4_regs[p][2], d[4], d[5]);
                    unpack8_nat((uint32_t)w4_regs[p][3], d[6], d[7]);
                }
                const int s = swz<BK>(row);
                *reinterpret_cast<int32x4 *>(base + row * BK + (((2 * q) ^ s) * 16)) =
                    int32x4{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
                *reinterpret_cast<int32x4 *>(base + row * BK + (((2 * q + 1) ^ s) * 16)) =
                    int32x4{(int)d[4], (int)d[5], (int)d[6], (int)d[7]};
            }
        }
    };

    // ---- accumulators -----------------------------------------------------
    AccT acc[FN][FM];
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[fn][fm][e] = 0;

    const int team = (KT == 1) ? 0 : wave / (WAVES_M * WAVES_N);
    const int wt = (KT == 1) ? wave : wave % (WAVES_M * WAVES_N);
    const int wm = wt % WAVES_M, wn = wt / WAVES_M;
    const int ks0 = team * KS_T;             // first k step of a stage that this wave multiplies
    const int lr = lane % 32;                // fragment row supplied by this lane
    const int lc = lane / 32;                // which 16-byte half of the 32-byte k step
    const int sw = swz<BK>(lr);              // wave and fragment offsets are multiples of 32 rows
    const int x_off = (wm * WM + lr) * BK;
    const int w_off = X_STAGE + (wn * WN + lr) * BKW;

    // Fragment loads and matrix-core steps of one 32-byte k step, in the order
    // the MFMAs consume them: a[0], every bx, then the remaining a.
    auto read_frags = [&](const uint8_t *sb, int ks, int32x4(&a)[FN], int32x4(&bx)[FM]) {
        const int p = (((ks + ks0) * 2 + lc) ^ sw) * 16;
        a[0] = *reinterpret_cast<const int32x4 *>(sb + w_off + p);
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) bx[fm] = *reinterpret_cast<const int32x4 *>(sb + x_off + fm * 32 * BK + p);
#pragma unroll
        for (int fn = 1; fn < FN; ++fn) a[fn] = *reinterpret_cast<const int32x4 *>(sb + w_off + fn * 32 * BK + p);
    };
    auto mfma_step = [&](const int32x4(&a)[FN], const int32x4(&bx)[FM]) {
        if constexpr (!PAIRED) {
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
                    if constexpr (XT == 2)
                        acc[fn][fm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a[fn]),
                                                                              __builtin_bit_cast(half8, bx[fm]),
                                                                              acc[fn][fm], 0, 0, 0);
                    else
                        acc[fn][fm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[fn], bx[fm], acc[fn][fm], 0, 0, 0);
        }
    };
    // Weight rows half as long as activation rows (PAIRED), told for FP16 activations; with INT8 activations and
    // INT4 weights a stage holds 128 values of K and every count of values below doubles.  A stage holds 64 values of K: 128 bytes (eight chunks) of an activation row, 64 bytes
    // (four chunks) of a weight row, four k steps of sixteen values.  Lane (row lr, half lc) reads weight
    // chunk 2*pair + lc once per pair of k steps: its first eight codes feed the first step of the pair, its
    // last eight the second.  The activations of the same values of K are chunk 4*pair + 2*lc + t for step
    // t of the pair, so every step reads one 16-byte activation chunk per row as before.
    const int sww = swz<BKW>(lr);
    auto read_x_paired = [&](const uint8_t *sb, int ks, int32x4(&bx)[FM]) {
        const int p = (((ks / 2) * 4 + 2 * lc + (ks & 1)) ^ sw) * 16;
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) bx[fm] = *reinterpret_cast<const int32x4 *>(sb + x_off + fm * 32 * BK + p);
    };
    int32x4 w_raw[FN];                       // the narrow weights of the next pair of k steps
    using WOp = typename std::conditional<A16, half8, int32x4>::type;
    WOp w_op[2][FN];                        // [step of the pair][fragment]: one set, rewritten once the
                                             // second step's MFMAs have been issued (register budget)
    auto read_w_paired = [&](const uint8_t *sb, int pair) {
        const int p = ((pair * 2 + lc) ^ sww) * 16;
#pragma unroll
        for (int fn = 0; fn < FN; ++fn) w_raw[fn] = *reinterpret_cast<const int32x4 *>(sb + w_off + fn * 32 * BKW + p);
    };
    // first (T = 0) or last (T = 1) eight bytes of w_raw -> the operands of that step of the pair (eight INT8
    // codes to FP16, or sixteen nibbles to INT8 times 16, both exact)
    auto convert_w_paired = [&](auto t_c) __attribute__((always_inline)) {
        constexpr int T = decltype(t_c)::value;
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
            if constexpr (A16) {
                w_op[T][fn] = cvt8_i8_f16((uint32_t)w_raw[fn][2 * T], (uint32_t)w_raw[fn][2 * T + 1]);
            } else {
                uint32_t d0, d1, d2, d3;
                unpack8_nat((uint32_t)w_raw[fn][2 * T], d0, d1);
                unpack8_nat((uint32_t)w_raw[fn][2 * T + 1], d2, d3);
                w_op[T][fn] = int32x4{(int)d0, (int)d1, (int)d2, (int)d3};
            }
    };
    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;
    // order of issue inside a step: one LDS read per MFMA while reads are left, then the conversion
    // spread over the remaining MFMAs
    auto pace_paired = [&](auto reads_c) __attribute__((always_inline)) {
        constexpr int READS = decltype(reads_c)::value;
        constexpr int NM = FN * FM;
        constexpr int VC = 10 * FN;                // VALU instructions of one conversion
        if constexpr (READS < NM) {
            constexpr int PER = (VC + NM - READS - 1) / (NM - READS);
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   // MFMA
                if (i < READS)
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);               // DS read
                else
                    __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);             // VALU
            }
        } else {                                   // small wave tiles: the reads outnumber the MFMAs
            constexpr int PER = (READS + NM - 1) / NM;
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, PER, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x002, VC, 0);
        }
    };
    using RX = std::integral_constant<int, FM>;          // a step that reads activation fragments only
    using RXW = std::integral_constant<int, FM + FN>;    // ... and the raw weights of the next pair
    auto mfma_step_paired = [&](const WOp(&a)[FN], const int32x4(&bx)[FM]) {
        if constexpr (PAIRED) {
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
                    if constexpr (A16)
                        acc[fn][fm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[fn], __builtin_bit_cast(half8, bx[fm]),
                                                                              acc[fn][fm], 0, 0, 0);
                    else
                        acc[fn][fm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[fn], bx[fm], acc[fn][fm], 0, 0, 0);
        }
    };
    // one LDS read after every (FN*FM)/(FN+FM) MFMAs
    auto interleave = [&]() {
        constexpr int per_read = (FN * FM) / (FN + FM) > 0 ? (FN * FM) / (FN + FM) : 1;
#pragma unroll
        for (int i = 0; i < FN + FM; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, per_read, 0);   // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);          // DS read
        }
    };

    float *col_scale = reinterpret_cast<float *>(smem + Cfg::kMain);
    float *col_bias = col_scale + BN;
    float *row_scale = col_bias + BN;

    // ---- main loop ----------------------------------------------------------
    // Stage kt lives in slot kt % NSTAGE.  During the last k step of stage kt every wave already holds
    // that step's fragments in registers, so after the barrier there the slot is free and receives
    // stage kt + NSTAGE, while the first fragments of stage kt + 1 are read under the last MFMAs.
    int32x4 a0[FN], b0[FM], a1[FN], b1[FM];
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s) {
        issue_direct(kt0 + s, s, s >= n_loc);
        if (STAGED_W && s < n_loc) {
            w4_fetch(kt0 + s, false);
            w4_store(s);
        }
    }
    // Scale prefetch (App. D reads both scale vectors before the product is complete): the
    // per-column weight-group scale and bias and the per-row token scale of this tile go to LDS.
    // They are requested after the first operand stages, and all three loads of a thread before
    // any of them is used, so that their round trip runs under the operand loads instead of in
    // front of them (it used to cost three dependent round trips before the first operand load).
    static_assert(BN <= NT && BM <= NT, "one scale element per thread");
    if constexpr (KSPLIT == 0) {
        const int c = threadIdx.x;
        int n = n0 + (c < BN ? c : 0);
        if (n > N - 1) n = N - 1;
        int m = m0 + (c < BM ? c : 0);
        if (m > M - 1) m = M - 1;
        const float sw_v = s_w[n / gs];
        // without a bias the load reads a valid dummy address: no branch around a load in flight
        const half_t b_v = *(bias != nullptr ? bias + n : reinterpret_cast<const half_t *>(s_w));
        const float st_v = A16 ? 1.0f : s_tok[m];         // FP16 activations carry no token scale
        if (c < BN) {
            col_scale[c] = sw_v;
            col_bias[c] = (bias != nullptr) ? (float)b_v : 0.0f;
        }
        if (c < BM) row_scale[c] = st_v;
    }
    if (!STAGED_W)
        wait_vmcnt<(NSTAGE - 1) * LPS>();      // stage 0 has landed; later stages may still be in flight
    else
        wait_vmcnt<0>();
    __syncthreads();
    if constexpr (PAIRED) {
        read_x_paired(smem, 0, b0);
        read_w_paired(smem, 0);
        convert_w_paired(T0{});
        convert_w_paired(T1{});
    } else {
        read_frags(smem, 0, a0, b0);
    }

    // One stage of K.  The last stage of the workgroup is a copy of its own (LAST = 1) without the
    // barrier, the refill and the read-ahead: were it a branch inside the loop, the paths with and
    // without the barrier would meet again in front of the last matrix-core step, and the compiler,
    // which tracks LDS reads in flight per path, would make that step wait for the reads issued after
    // the barrier although its operands were read long before it.
    auto stage = [&](int kt, auto last_c) __attribute__((always_inline)) {
        constexpr bool LAST = decltype(last_c)::value;
        const uint8_t *sb = smem + (kt % NSTAGE) * STAGE;
        const uint8_t *sn = smem + ((kt + 1) % NSTAGE) * STAGE;
        if constexpr (PAIRED) {
            // k steps 0..3 = (pair 0, step 0), (pair 0, step 1), (pair 1, step 0), (pair 1, step 1).  The second
            // step of a pair reads the raw weights of the next pair and converts their first half (whose
            // registers the first step has finished with) under its own MFMAs; the first step of the next
            // pair converts the second half under its MFMAs.  One set of converted operands is enough.
            read_x_paired(sb, 1, b1);
            mfma_step_paired(w_op[0], b0);
            convert_w_paired(T1{});
            pace_paired(RX{});
            read_x_paired(sb, 2, b0);
            read_w_paired(sb, 1);
            mfma_step_paired(w_op[1], b1);
            convert_w_paired(T0{});
            pace_paired(RXW{});
            read_x_paired(sb, 3, b1);
            mfma_step_paired(w_op[0], b0);
            convert_w_paired(T1{});
            pace_paired(RX{});
            if constexpr (!LAST) {
                wait_vmcnt<(NSTAGE - 2) * LPS>();         // stage kt+1 has landed
                lds_barrier();
                issue_direct(kt0 + kt + NSTAGE, kt % NSTAGE, kt + NSTAGE >= n_loc);
                read_x_paired(sn, 0, b0);
                read_w_paired(sn, 0);
            }
            mfma_step_paired(w_op[1], b1);
            if constexpr (!LAST) {
                convert_w_paired(T0{});
                pace_paired(RXW{});
            }
            return;
        }
#pragma unroll
        for (int ks = 0; ks < KS_T; ++ks) {
            int32x4(&ca)[FN] = (ks & 1) ? a1 : a0;
            int32x4(&cb)[FM] = (ks & 1) ? b1 : b0;
            int32x4(&na)[FN] = (ks & 1) ? a0 : a1;
            int32x4(&nb2)[FM] = (ks & 1) ? b0 : b1;
            if (ks + 1 < KS_T) {
                read_frags(sb, ks + 1, na, nb2);
                mfma_step(ca, cb);
                interleave();
            } else {
                if constexpr (!LAST) {
                    if (!STAGED_W)
                        wait_vmcnt<(NSTAGE - 2) * LPS>();     // stage kt+1 has landed
                    else
                        wait_vmcnt<0>();
                    // Weights that pass through registers (INT4 nibbles, INT8 -> FP16): the registers fetched
                    // at the previous boundary have had a whole stage to arrive and share the wait above;
                    // their slot was freed at that boundary.  (Placed at the start of the stage, as before,
                    // the store waited for loads issued one k step earlier, a full memory latency per stage.)
                    if (STAGED_W && kt >= 1 && kt - 1 + NSTAGE < n_loc) w4_store((kt - 1) % NSTAGE);
                    lds_barrier();
                    issue_direct(kt0 + kt + NSTAGE, kt % NSTAGE, kt + NSTAGE >= n_loc);
                    if (STAGED_W) w4_fetch(kt0 + kt + NSTAGE, kt + NSTAGE >= n_loc);
                    read_frags(sn, 0, na, nb2);
                }
                mfma_step(ca, cb);
                if constexpr (!LAST) interleave();     // the first fragments of the next stage arrive under these MFMAs
            }
        }
    };
    static_assert(KS_T % 2 == 0, "a stage starts on the first fragment set");
    for (int kt = 0; kt < n_loc - 1; ++kt)     // kt counts this workgroup's stages; kt0 + kt is the stage of K
        stage(kt, std::false_type{});
    stage(n_loc - 1, std::true_type{});

    // ---- epilogue ---------------------------------------------------------
    // acc[fn][fm][v]: output column n = wn*WN + fn*32 + 8*(v/4) + 4*(lane/32) + v%4,
    //                 token row     m = wm*WM + fm*32 + lane%32.
    if constexpr (KSPLIT == 1) {
        // K split: the raw accumulators of this range of K go to partial[split][M][N]; the second
        // kernel adds the splits in order and applies scales, bias and activation.  Each wave turns its
        // WM x WN block through a wave-private LDS buffer (rows padded by 16 bytes against bank
        // conflicts; the LDS operations of one wave complete in order) so that it leaves as whole row
        // segments of WN * 4 bytes instead of one 16-byte piece per row and lane.
        constexpr int PROW = WN + 4;                  // ints per padded row
        static_assert(NW * WM * PROW * 4 <= NSTAGE * STAGE, "the partial tile is staged in the stage ring");
        static_assert((WM * WN / 4) % 64 == 0, "whole store instructions per wave");
        __syncthreads();                              // all reads of the last stage are done
        int32_t *pt = reinterpret_cast<int32_t *>(smem) + wave * (WM * PROW);
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if constexpr (A16)
                            v[e] = __float_as_int(acc[fn][fm][4 * q + e]);
                        else
                            v[e] = acc[fn][fm][4 * q + e];
                    }
                    *reinterpret_cast<int32x4 *>(pt + (fm * 32 + lr) * PROW + fn * 32 + 8 * q + 4 * lc) = v;
                }
            }
        }
        int32_t *mine = partial + (size_t)split * M * N;
        constexpr int CPW = WN / 4;                   // 16-byte pieces per row of the wave's block
#pragma unroll
        for (int i = 0; i < WM * CPW / 64; ++i) {
            const int row = (i * 64 + lane) / CPW, c = (i * 64 + lane) % CPW;
            const int32x4 v = *reinterpret_cast<const int32x4 *>(pt + row * PROW + c * 4);
            const int m = m0 + wm * WM + row, n = n0 + wn * WN + c * 4;
            if (m < M && n < N) *reinterpret_cast<int32x4 *>(mine + (size_t)m * N + n) = v;
        }
        return;
    }
    __syncthreads();                          // all reads of the last stage are done; LDS is reused below
    if constexpr (KT == 2) {
        // The two teams hold partial products of the same tile.  Each wave hands the half of its 32-row
        // blocks that its partner wave (same place in the other team) will finish to LDS, one 16-byte piece
        // per lane and group of four registers, and adds the partner's pieces for the half it keeps.
        // Integer sums do not depend on the order; the fp32 ones are one addition of the same two
        // numbers on either side.
        constexpr int HALF = FM / 2;
        int32x4 *xb = reinterpret_cast<int32x4 *>(smem + Cfg::kXchg);
        constexpr int PER_WAVE = HALF * FN * 4 * 64;          // 16-byte pieces per wave
        auto hand_over = [&](auto lo_c) __attribute__((always_inline)) {
            constexpr int LO = decltype(lo_c)::value;         // first block handed over
#pragma unroll
            for (int fm = 0; fm < HALF; ++fm)
#pragma unroll
                for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        int32x4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if constexpr (A16)
                                v[e] = __float_as_int(acc[fn][LO + fm][4 * q + e]);
                            else
                                v[e] = acc[fn][LO + fm][4 * q + e];
                        }
                        xb[wave * PER_WAVE + ((fm * FN + fn) * 4 + q) * 64 + lane] = v;
                    }
        };
        auto take_over = [&](auto lo_c) __attribute__((always_inline)) {
            constexpr int LO = decltype(lo_c)::value;         // first block kept
            const int partner = (wave + WAVES_M * WAVES_N) % (2 * WAVES_M * WAVES_N);
#pragma unroll
            for (int fm = 0; fm < HALF; ++fm)
#pragma unroll
                for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int32x4 v = xb[partner * PER_WAVE + ((fm * FN + fn) * 4 + q) * 64 + lane];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if constexpr (A16)
                                acc[fn][LO + fm][4 * q + e] += __int_as_float(v[e]);
                            else
                                acc[fn][LO + fm][4 * q + e] += v[e];
                        }
                    }
        };
        if (team == 0)
            hand_over(std::integral_constant<int, HALF>{});   // team 0 keeps blocks 0 .. HALF-1
        else
            hand_over(std::integral_constant<int, 0>{});
        __syncthreads();
        if (team == 0)
            take_over(std::integral_constant<int, 0>{});
        else
            take_over(std::integral_constant<int, HALF>{});
    }
    constexpr int OROW = Cfg::kEpiRow;
    uint8_t *ot = smem + wave * (32 * OROW);  // wave-private: 32 rows of this wave's columns
    const int mw = m0 + wm * WM;              // first token row of this wave
    const int nw = n0 + wn * WN;              // first output column of this wave
    constexpr int LPR = WN * 2 / 16;          // lanes per output row (16 bytes each)
    static_assert((32 * LPR) % 64 == 0, "the 32-row block must be a whole number of store instructions");
    float rmax[FM];                           // QOUT: max |g| of this lane's token rows
    unsigned gen_raw = 0;                     // QOUT: generation of this launch, back before it is needed
    if constexpr (QOUT == 1)
        gen_raw = __hip_atomic_load(q_ctl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // The column scales and biases of this wave's columns, read once where the registers allow it
    // (they do not depend on the row).
    constexpr bool HOIST = FN <= 2 && QOUT == 0;      // the in-kernel quantizer keeps the accumulators live longer
    // The four consecutive columns of a lane's register group lie in one weight group (a group is a
    // multiple of 16 columns and the four start at a multiple of 4), so one scale serves all four.
    float sc_all[HOIST ? FN : 1][4];
    float4 cb_all[HOIST ? FN : 1][4];
    if constexpr (HOIST) {
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int nl = fn * 32 + 8 * q + 4 * lc;
                sc_all[fn][q] = col_scale[wn * WN + nl];
                cb_all[fn][q] = *reinterpret_cast<const float4 *>(col_bias + wn * WN + nl);
            }
    }
    // PLAIN = no activation and no accumulator tap, decided once for the whole epilogue: with the two
    // (wave-uniform) tests inside the loops every group of four values was a basic block of its own
    // and its LDS round trip could not overlap the arithmetic of its neighbours.
    auto rows_pass = [&](auto plain_c, auto lo_c, auto hi_c) __attribute__((always_inline)) {
        constexpr bool PLAIN = decltype(plain_c)::value;
        constexpr int FM_LO = decltype(lo_c)::value, FM_HI = decltype(hi_c)::value;   // the 32-row blocks this wave finishes
#pragma unroll
        for (int fm = FM_LO; fm < FM_HI; ++fm) {
            rmax[fm] = 0.0f;
            const float st = row_scale[wm * WM + fm * 32 + lr];
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nl = fn * 32 + 8 * q + 4 * lc;
                    const float sc = HOIST ? sc_all[HOIST ? fn : 0][q] : col_scale[wn * WN + nl];
                    const float4 cb = HOIST ? cb_all[HOIST ? fn : 0][q]
                                            : *reinterpret_cast<const float4 *>(col_bias + wn * WN + nl);
                    int32x4 v = {0, 0, 0, 0};
                    float fv[4];
                    if constexpr (A16) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) fv[e] = acc[fn][fm][4 * q + e];
                    } else {
                        v = int32x4{acc[fn][fm][4 * q], acc[fn][fm][4 * q + 1], acc[fn][fm][4 * q + 2],
                                    acc[fn][fm][4 * q + 3]};
                        if (WBITS == 4) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] >>= 4;   // exact: every product carried the factor 16
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) fv[e] = (float)v[e];
                    }
                    // one rounded product of the two scales, then one fused multiply-add: written out so
                    // that every instantiation of this epilogue rounds alike (left to the compiler, one
                    // copy was contracted and another was not, one FP16 step apart on a few values)
                    const float ss = st * sc;
                    float f[4] = {__builtin_fmaf(fv[0], ss, cb.x), __builtin_fmaf(fv[1], ss, cb.y),
                                  __builtin_fmaf(fv[2], ss, cb.z), __builtin_fmaf(fv[3], ss, cb.w)};
                    if constexpr (!PLAIN) apply_activation_n<4>(f, act);    // act is wave-uniform
                    half4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // the fp32 value is rounded to fp32 first and to FP16 second in every instantiation:
                        // without this the compiler merges the multiply-add and the conversion of some
                        // values into one mixed-precision instruction with a single rounding, and the
                        // kernel that quantizes its output would not give the bits of the plain one
                        asm("" : "+v"(f[e]));
                        o[e] = (half_t)f[e];
                    }
                    if (QOUT == 0 || out != nullptr) *reinterpret_cast<half4 *>(ot + lr * OROW + nl * 2) = o;
                    if constexpr (!PLAIN && !A16) {
                        if (acc_out != nullptr) {
                            const int m = mw + fm * 32 + lr;
                            if (m < M && nw + nl < N)
                                *reinterpret_cast<int32x4 *>(acc_out + (size_t)m * N + nw + nl) = v;
                        }
                    }
                    if constexpr (QOUT == 1) {
                        // the accumulator registers now hold the output as rounded to FP16: the codes
                        // below are those of the stored tensor
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float g = (float)o[e];
                            acc[fn][fm][4 * q + e] = __float_as_int(g);
                            rmax[fm] = fmaxf(rmax[fm], fabsf(g));
                        }
                    }
                }
            }
            // The wave reads back its own 32 rows (LDS operations of one wave complete in order) and
            // stores whole row segments.
            if (QOUT == 0 || out != nullptr) {
#pragma unroll
                for (int i = 0; i < 32 * LPR / 64; ++i) {
                    const int row = (i * 64 + lane) / LPR;
                    const int col = ((i * 64 + lane) % LPR) * 8;
                    const int32x4 v = *reinterpret_cast<const int32x4 *>(ot + row * OROW + col * 2);
                    const int m = mw + fm * 32 + row;
                    const int n = nw + col;
                    // Streaming (non-temporal) stores: nothing in this kernel reads the output again, and lines
                    // that do not linger in the L2 need no write-back when the kernel ends (4096x4096x1024:
                    // 25.3 -> 23.2 us alone, 23.5 -> 23.0 us inside the feed-forward chain).
                    if (m < M && n < N)
                        __builtin_nontemporal_store(v, reinterpret_cast<int32x4 *>(out + (size_t)m * N + n));
                }
            }
        }
    };
    const bool plain = QOUT == 0 && act == 0 && acc_out == nullptr;
    using I0 = std::integral_constant<int, 0>;
    using IH = std::integral_constant<int, FM / 2>;
    using IF = std::integral_constant<int, FM>;
    if constexpr (KT == 1) {
        if (plain)
            rows_pass(std::true_type{}, I0{}, IF{});
        else
            rows_pass(std::false_type{}, I0{}, IF{});
    } else {
        if (team == 0) {
            if (plain)
                rows_pass(std::true_type{}, I0{}, IH{});
            else
                rows_pass(std::false_type{}, I0{}, IH{});
        } else {
            if (plain)
                rows_pass(std::true_type{}, IH{}, IF{});
            else
                rows_pass(std::false_type{}, IH{}, IF{});
        }
    }

    if constexpr (QOUT == 1) {
        // ---- token-wise quantization of the output rows from registers (App. A.2) ----
        // A row of g spans the tiles_n tiles of this band.  Row maxima: lane pair -> the waves along
        // N (LDS) -> the band (slots in device memory).  Columns past N repeat column N-1 and rows
        // past M repeat row M-1 (clamped loads), so they never raise a maximum.
        float *wave_max = row_scale + BM;              // [WAVES_N][BM]
        float *row_inv = wave_max + WAVES_N * BM;      // [BM]
        const int tid = threadIdx.x;
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
            rmax[fm] = fmaxf(rmax[fm], __shfl_xor(rmax[fm], 32));
            if (lc == 0) wave_max[wn * BM + wm * WM + fm * 32 + lr] = rmax[fm];
        }
        __syncthreads();
        const unsigned tag = gen_raw + 1u;             // never 0: untouched slots carry tag 0
        if (tid < BM) {
            float a = wave_max[tid];
#pragma unroll
            for (int w = 1; w < WAVES_N; ++w) a = fmaxf(a, wave_max[w * BM + tid]);
            // Publish this tile's maxima, then collect the band's: one store and, when the other
            // tiles are already there, one round of loads.  Maxima are compared as integers (the
            // bits of non-negative floats order like the floats).  The wait is bounded.  A thread
            // whose wait ran out counts itself in the control block, overwrites its slot with a
            // NaN (tiles that arrive later then see it as the maximum) and takes NaN as the row
            // maximum: its scale is NaN and its codes are -128, which the quantizer never produces.
            unsigned long long *band = q_slots + (size_t)tm * tiles_n * BM + tid;
            __hip_atomic_store(band + (size_t)tn * BM, ((unsigned long long)tag << 32) | __float_as_uint(a),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            constexpr int QB = 16;                     // slots fetched per round
            unsigned spins = 0;
            unsigned abits = __float_as_uint(a);
            for (int j0 = 0; j0 < tiles_n; j0 += QB) {
                while (true) {
                    unsigned long long v[QB];
#pragma unroll
                    for (int u = 0; u < QB; ++u) {
                        const int j = (j0 + u < tiles_n) ? j0 + u : tiles_n - 1;
                        v[u] = __hip_atomic_load(band + (size_t)j * BM, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    bool all = true;
                    unsigned mx = abits;
#pragma unroll
                    for (int u = 0; u < QB; ++u) {
                        all = all && (unsigned)(v[u] >> 32) == tag;
                        const unsigned b = (unsigned)v[u];
                        mx = b > mx ? b : mx;
                    }
                    if (all) {
                        abits = mx;
                        break;
                    }
                    if (++spins > kQuantSpinLimit) {
                        __hip_atomic_fetch_add(q_ctl + 2, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __hip_atomic_store(band + (size_t)tn * BM, ((unsigned long long)tag << 32) | kPoisonBits,
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        abits = kPoisonBits;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
                }
                if (abits >= kPoisonBits) break;
            }
            float scale, inv;
            if (abits >= kPoisonBits) {
                scale = __uint_as_float(kPoisonBits);
                inv = __uint_as_float(kPoisonBits);
            } else {
                quant_scales(__uint_as_float(abits), 127.0f, scale, inv);
            }
            row_inv[tid] = inv;
            if (tn == 0 && m0 + tid < M) q_scale_out[m0 + tid] = scale;
        }
        __syncthreads();
        // This workgroup has read its band.  The count comes back while the codes are written; the
        // workgroup that completes it ends the launch's generation (below).
        unsigned done_before = 0;
        if (tid == 0)
            done_before = __hip_atomic_fetch_add(q_ctl + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // Codes: four consecutive columns per lane -> one dword of the BM x BN code tile in LDS (the
        // stage ring is free now), 16-byte chunks XOR-swizzled by row so that the 32 rows of a
        // fragment hit different banks; then every row leaves as one contiguous segment.
        constexpr int QCH = BN / 16;                   // 16-byte chunks per row of the code tile
        uint8_t *ct = smem;
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
            const int row = wm * WM + fm * 32 + lr;
            const float inv = row_inv[row];
            const bool poisoned = __float_as_uint(inv) == kPoisonBits;   // the wait of this row ran out
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = wn * WN + fn * 32 + 8 * q + 4 * lc;
                    uint32_t d = pack4_code_bits(
                        quant_code_bits(__int_as_float(acc[fn][fm][4 * q]), inv),
                        quant_code_bits(__int_as_float(acc[fn][fm][4 * q + 1]), inv),
                        quant_code_bits(__int_as_float(acc[fn][fm][4 * q + 2]), inv),
                        quant_code_bits(__int_as_float(acc[fn][fm][4 * q + 3]), inv));
                    if (poisoned) d = 0x80808080u;
                    *reinterpret_cast<uint32_t *>(ct + row * BN + (((col / 16) ^ (row & (QCH - 1))) * 16) + col % 16) = d;
                }
            }
        }
        __syncthreads();
        for (int idx = tid; idx < BM * QCH; idx += NT) {
            const int row = idx / QCH, c = idx % QCH;
            const int32x4 v = *reinterpret_cast<const int32x4 *>(ct + row * BN + ((c ^ (row & (QCH - 1))) * 16));
            const int m = m0 + row, n = n0 + c * 16;
            if (m < M && n < N) *reinterpret_cast<int32x4 *>(q_out + (size_t)m * N + n) = v;
        }
        if (tid == 0 && done_before == gridDim.x - 1u) {
            __hip_atomic_store(q_ctl + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned next = gen_raw + 1u;        // the tag, next + 1, must never be 0
            __hip_atomic_store(q_ctl, next != 0xffffffffu ? next : 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
#endif
}


namespace {

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NSTAGE, int WBITS, int XT = 0, int QOUT = 0,
          int KSPLIT = 0, int KT = 1>
hipError_t launch_tile_t(const GemmArgs &a, hipStream_t st, int k_splits = 1) {
    using Cfg = TileCfg<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, KT, XT>;
    constexpr size_t lds = QOUT ? Cfg::kLdsQ : Cfg::kLds;
    static std::atomic<uint64_t> configured{0};
    const void *kernel = reinterpret_cast<const void *>(
        &gemm_tile_kernel<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, WBITS, XT, QOUT, KSPLIT, KT>);
    if (hipError_t e = ensure_dynamic_lds(kernel, lds, configured); e != hipSuccess) return e;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    if (KSPLIT == 0 && k_splits != 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, WBITS, XT, QOUT, KSPLIT, KT>),
                       dim3(tiles_m * tiles_n * k_splits), dim3(Cfg::kThreads), lds, st, a.xq, a.s_tok,
                       reinterpret_cast<const uint8_t *>(a.wq), a.s_w, a.N / a.groups,
                       reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K, reinterpret_cast<half_t *>(a.out),
                       a.acc_out, tiles_m, tiles_n, a.act, a.q_out, a.q_scale_out, k_splits,
                       KSPLIT ? reinterpret_cast<int32_t *>(ws_partials(a.workspace)) : nullptr,
                       QOUT ? ws_slots(a.workspace) : nullptr, QOUT ? ws_control(a.workspace) : nullptr);
    return hipGetLastError();
}

// Second kernel of the K split: adds the partial products of the splits (in split order, so that the
// fp32 sums of the FP16-activation product do not depend on timing) and applies the epilogue of the
// tiled kernel: acc * (s_tok[row] * s_w[group]) + bias, activation, one rounding to FP16.  One thread
// per four consecutive columns; INT4 products carry the factor 16 of the nibble unpack until here.
template <int XT>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const int32x4 *__restrict__ partial, int k_splits,
                                                            const float *__restrict__ s_tok,
                                                            const float *__restrict__ s_w, int gs,
                                                            const half_t *__restrict__ bias, int M, int N,
                                                            half4 *__restrict__ out, int32x4 *__restrict__ acc_out,
                                                            int act, int shift) {
    const int nq = N >> 2;
    const long total = (long)M * nq;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int m = (int)(i / nq);
        const int n = (int)(i - (long)m * nq) * 4;
        float fv[4];
        int32x4 sum = {0, 0, 0, 0};
        if constexpr (XT == 1) {
            float32x4 fs = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 4
            for (int s = 0; s < k_splits; ++s) fs += __builtin_bit_cast(float32x4, partial[(long)s * total + i]);
#pragma unroll
            for (int e = 0; e < 4; ++e) fv[e] = fs[e];
        } else {
#pragma unroll 4
            for (int s = 0; s < k_splits; ++s) sum += partial[(long)s * total + i];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sum[e] >>= shift;                     // exact: every INT4 product carried the factor 16
                fv[e] = (float)sum[e];
            }
            if (acc_out != nullptr) acc_out[i] = sum;
        }
        const float st = (XT == 1) ? 1.0f : s_tok[m];
        const float sc = s_w[n / gs];
        float f[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float cb = (bias != nullptr) ? (float)bias[n + e] : 0.0f;
            f[e] = __builtin_fmaf(fv[e], st * sc, cb);
        }
        apply_activation_n<4>(f, act);
        half4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (half_t)f[e];
        out[i] = o;
    }
}

// K splits of the 128x128-tile schedule for a shape whose tiles leave most compute units idle: at
// most as many as fill the chip once, at least four stages of K each, at most sixteen, and among
// those the count with the lowest modelled time; 1 = no split pays.  The model, fitted to
// measurements at 130 to 1024 tokens (microseconds): a tile over K takes 4.5 + u per 1024 bytes of
// an activation row (u = 4.0 for INT8 activations, 5.2 for FP16 ones); the K split adds the second
// kernel's launch, 3, and 0.5 per MB of partial products written and read back.
int tile_splits(int M, int N, int K, int x_bytes) {
    const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
    const int nkt = (K * x_bytes + 127) / 128;
    if (tiles > 128 || nkt < 8) return 1;
    int ks_max = (int)(256 / tiles);
    if (ks_max > nkt / 4) ks_max = nkt / 4;
    if (ks_max > 16) ks_max = 16;
    const double unit = (x_bytes == 1) ? 4.0 : 5.2;
    const double k_units = (double)K * x_bytes / 1024.0;
    const double whole = 4.5 + unit * k_units;
    int best = 1;
    double best_t = 0.9 * whole;                      // a split has to win by a tenth
    for (int ks = 2; ks <= ks_max; ++ks) {
        const double t = 7.5 + unit * k_units / ks + 0.5e-6 * ks * (double)M * N * 4.0;
        if (t < best_t) {
            best_t = t;
            best = ks;
        }
    }
    return best;
}

// Tile edge of the schedule that quantizes its output in the kernel: 256 where the plain call
// would use it or where 128x128 tiles would outnumber what eight-wave workgroups hold at once.
int quant_tile_edge(int M, int N) {
    const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256);
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    return (t256 >= 160 || t128 > 384) ? 256 : 128;
}

}  // namespace

// block: 256 = 256x256 tile, eight waves; 256192 = 256x192 tile, eight waves (4 x 2, wave tile 64 x 96);
//        192 = 256x128 tile, four waves, two workgroups per CU;
//        128 = 128x128 tile, eight waves on a deep ring of 128-byte stages (two waves per SIMD); INT8 weights: two K teams.
hipError_t launch_gemm_tile(const GemmArgs &a, int block, hipStream_t st) {
    if (block == 256) {
        if (a.w_bits == 8) return launch_tile_t<256, 256, 2, 4, 128, 2, 8>(a, st);
        return launch_tile_t<256, 256, 2, 4, 128, 2, 4>(a, st);
    }
    if (block == 256192) {
        if (a.w_bits == 8) return launch_tile_t<256, 192, 4, 2, 128, 2, 8>(a, st);
        return launch_tile_t<256, 192, 4, 2, 128, 2, 4>(a, st);
    }
    if (block == 192) {
        if (a.w_bits == 8) return launch_tile_t<256, 128, 2, 2, 64, 3, 8>(a, st);
        return launch_tile_t<256, 128, 2, 2, 64, 3, 4>(a, st);
    }
    // INT8 weights: two K teams of 2 x 2 waves (wave tile 64 x 64); measured 5-8 % ahead of eight waves side by
    // side on 4096x1024x4096 and 2048x2048x8192, level on 2048x2048x2048.  INT4 weights measured 2-3 % slower with
    // teams (the nibble unpack already fills the stage boundary) and keep the 2 x 4 layout, with the nibbles
    // packed in LDS (XT = 3): these tiles wait for their operand loads, and half the weight bytes measured
    // 5-14 % faster (2048x2048x2048 13.5 -> 12.8 us, 4096x1024x4096 27.1 -> 23.7 us).  On 256 x 256 tiles, which
    // run at the chip's power limit, the register-side unpack measured 5 % slower than unpacking on the way
    // into LDS (4096x16384x4096 233 -> 245 us), so they keep that.
    if (a.w_bits == 8) return launch_tile_t<128, 128, 2, 2, 128, 4, 8, 0, 0, 0, 2>(a, st);
    return launch_tile_t<128, 128, 2, 4, 128, 4, 4, 3>(a, st);
}

// The 128x128-tile schedule with K split over workgroups and a second kernel for the epilogue: for
// token counts above the streaming schedules' whose tiles would occupy less than half the chip.
// The partial products go to the partial-sum part of a.workspace (gemm_tile_split_workspace() bytes in all).
int gemm_tile_splits(int M, int N, int K) {
    // the streaming schedules keep up to 64 tokens, and up to 128 where K is short (measured at 72 to 128
    // tokens, K split against streaming: 4096x4096 15.2 vs 17 us, 1024x4096 11.3 vs 13 us, 2048x2048 a tie)
    if ((K % 256) == 0 && (M <= 64 || (M <= 128 && K < 4096))) return 1;
    return tile_splits(M, N, K, 1);
}

size_t gemm_tile_split_workspace(int M, int N, int K) {
    const int ks = gemm_tile_splits(M, N, K);
    return ks > 1 ? kWsFixedBytes + (size_t)ks * M * N * sizeof(int32_t) : 0;
}

namespace {
template <int XT>
hipError_t launch_splitk_finish(const GemmArgs &a, int k_splits, hipStream_t st) {
    const long total = (long)a.M * (a.N / 4);
    long blocks = (total + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL((splitk_finish_kernel<XT>), dim3((unsigned)blocks), dim3(256), 0, st,
                       reinterpret_cast<const int32x4 *>(ws_partials(a.workspace)), k_splits, a.s_tok, a.s_w,
                       a.N / a.groups,
                       reinterpret_cast<const half_t *>(a.bias), a.M, a.N, reinterpret_cast<half4 *>(a.out),
                       reinterpret_cast<int32x4 *>(a.acc_out), a.act, a.w_bits == 4 ? 4 : 0);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_gemm_tile_splitk(const GemmArgs &a, hipStream_t st) {
    const int ks = gemm_tile_splits(a.M, a.N, a.K);
    if (ks < 2 || a.workspace == nullptr ||
        a.workspace_bytes < kWsFixedBytes + (size_t)ks * a.M * a.N * sizeof(int32_t))
        return hipErrorInvalidValue;
    // INT4 weights packed in LDS (XT = 3), as in the unsplit 128 x 128 schedule: 4096x16384 at 256 / 512 tokens
    // 38.6 -> 35.3 / 56.4 -> 52.0 us
    hipError_t e = (a.w_bits == 8) ? launch_tile_t<128, 128, 2, 4, 128, 4, 8, 0, 0, 1>(a, st, ks)
                                   : launch_tile_t<128, 128, 2, 4, 128, 4, 4, 3, 0, 1>(a, st, ks);
    if (e != hipSuccess) return e;
    return launch_splitk_finish<0>(a, ks, st);
}

// The tiled GeMM with the token-wise quantization of its output inside the kernel (a.q_out,
// a.q_scale_out; a.out optional).  The tiles of a band of token rows wait for each other.  Workgroups
// are started in id order and the tiles of a band have consecutive ids, so the oldest unfinished band
// of a launch has all its tiles running as soon as the launch holds a band's worth of compute units
// (one workgroup of these kernels occupies a compute unit); a band is therefore limited to a quarter
// of the compute units the device reports, which also leaves room for up to four such launches side
// by side on different streams.  Every (tile, row) needs an exchange slot of the workspace.
bool gemm_tile_quant_supported(int M, int N, size_t workspace_bytes) {
    if (workspace_bytes < kWsFixedBytes) return false;
    const int edge = quant_tile_edge(M, N);
    const int tiles_m = (M + edge - 1) / edge, tiles_n = (N + edge - 1) / edge;
    return tiles_n <= compute_units() / 4 && (long)tiles_m * tiles_n * edge <= kMaxQuantSlots;
}

hipError_t launch_gemm_tile_quant(const GemmArgs &a, hipStream_t st) {
    if (a.workspace == nullptr || !gemm_tile_quant_supported(a.M, a.N, a.workspace_bytes) || a.q_out == nullptr ||
        a.q_scale_out == nullptr)
        return hipErrorInvalidValue;
    if (quant_tile_edge(a.M, a.N) == 256) {
        if (a.w_bits == 8) return launch_tile_t<256, 256, 2, 4, 128, 2, 8, 0, 1>(a, st);
        return launch_tile_t<256, 256, 2, 4, 128, 2, 4, 0, 1>(a, st);
    }
    if (a.w_bits == 8) return launch_tile_t<128, 128, 2, 4, 128, 4, 8, 0, 1>(a, st);
    return launch_tile_t<128, 128, 2, 4, 128, 4, 4, 0, 1>(a, st);
}

// Compute units of the current device, asked once per device; 256 if no device answers.
int compute_units() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return 256;
    }
    std::atomic<int> &slot = cached[dev & 63];
    int v = slot.load(std::memory_order_relaxed);
    if (v > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    slot.store(v, std::memory_order_relaxed);
    return v;
}

// Zeroes the control words, the arrival counters and the exchange slots of a workspace.
__global__ __launch_bounds__(256) void workspace_fill_kernel(int32x4 *p, long n) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) p[i] = int32x4{0, 0, 0, 0};
}

hipError_t launch_workspace_init(void *ws, hipStream_t st) {
    const long n = (long)(kWsFixedBytes / 16);
    hipLaunchKernelGGL(workspace_fill_kernel, dim3(1024), dim3(256), 0, st, reinterpret_cast<int32x4 *>(ws), n);
    return hipGetLastError();
}

// K splits of the FP16-activation call on the tiled schedule (1: none) and the workspace they need.
int gemm_a16_tile_splits(int M, int N, int K) { return tile_splits(M, N, K, 2); }

size_t gemm_a16_tile_split_workspace(int M, int N, int K) {
    const int ks = tile_splits(M, N, K, 2);
    return ks > 1 ? kWsFixedBytes + (size_t)ks * M * N * sizeof(float) : 0;
}

// FP16 activations x INT8 weights on the tiled schedules.  The argument block is the
// INT8 one with xq pointing at the FP16 activations and no token scales.
hipError_t launch_gemm_a16_tile(const A16Args &a16, hipStream_t st) {
    GemmArgs a;
    a.xq = reinterpret_cast<const int8_t *>(a16.x);
    a.s_tok = nullptr;
    a.wq = a16.wq; a.s_w = a16.s_w; a.groups = a16.groups; a.bias = a16.bias;
    a.M = a16.M; a.N = a16.N; a.K = a16.K; a.out = a16.out; a.acc_out = nullptr;
    a.workspace = a16.workspace; a.workspace_bytes = a16.workspace_bytes; a.w_bits = 8; a.act = 0;
    // few tiles against a long K: split K (fp32 partials, added in split order by the second kernel)
    const int ks = tile_splits(a.M, a.N, a.K, 2);
    if (ks > 1 && a.workspace != nullptr &&
        a.workspace_bytes >= kWsFixedBytes + (size_t)ks * a.M * a.N * sizeof(float)) {
        if (hipError_t e = launch_tile_t<128, 128, 2, 4, 128, 4, 8, 1, 0, 1>(a, st, ks); e != hipSuccess) return e;
        return launch_splitk_finish<1>(a, ks, st);
    }
    // the tile is chosen like the INT8 call's: rounds of tiles x area x a factor per tile shape
    const long rows256 = (a.M + 255) / 256;
    auto rounds = [](long tiles) { return (tiles + 255) / 256; };
    const long c256 = rounds(rows256 * ((a.N + 255) / 256)) * 65536 * 100;
    const long c192 = rounds(rows256 * ((a.N + 191) / 192)) * 49152 * 115;
    const long c128 = rounds((long)((a.M + 127) / 128) * ((a.N + 127) / 128)) * 16384 * 185;
    if (c128 <= c256 && c128 <= c192) return launch_tile_t<128, 128, 2, 4, 128, 4, 8, 1>(a, st);
    // the 256x192 tile keeps its weights FP16 in LDS (XT = 2): with three weight fragments per wave the
    // register-side conversion made the compiler copy the accumulators every stage
    if (c192 < c256) return launch_tile_t<256, 192, 4, 2, 128, 2, 8, 2>(a, st);
    return launch_tile_t<256, 256, 2, 4, 128, 2, 8, 1>(a, st);
}

}  // namespace zq
