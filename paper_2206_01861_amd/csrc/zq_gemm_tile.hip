// LDS-tiled INT8 GeMM with the dequantization epilogue for large token counts
// (Sec. 4.3 "INT8 GeMM"; App. D "Dequantization Associated with GeMM
// Schedule").  Bound by the INT8 matrix cores.
//
// A 256-thread workgroup (2 x 2 waves) owns a BM x BN output tile.  Per
// 128-byte step of K both operand tiles go from global memory straight into
// LDS with 16-byte direct loads (no register staging), double buffered; rows
// are 128 bytes with their 16-byte chunks XOR-swizzled so that the
// ds_read_b128 of a matrix-core fragment (32 rows, one chunk) is free of bank
// conflicts.  Each wave computes (BN/2) x (BM/2) with v_mfma_i32_32x32x32_i8,
// the weight fragment as the first operand, so every group of four accumulator
// registers runs along the output columns.  The epilogue scales the INT32
// accumulators by s_tok[row] * s_w[group], adds the bias, rounds to FP16,
// transposes the wave's tile through LDS (free after the main loop) and writes
// rows of 256 contiguous bytes.  INT4 weights are unpacked to INT8 (times 16)
// on their way into LDS and the factor is shifted out of the accumulator.
//
// Workgroup ids are remapped so that the workgroups an XCD receives
// (round-robin by id) cover a compact block of tiles and share operand panels
// in that XCD's L2.
#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

namespace {

constexpr uint32_t kRsrcFlags = 0x00020000u;
typedef __attribute__((address_space(3))) void lds_void;

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

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

}  // namespace

template <int BM, int BN, int WBITS>
__global__ __launch_bounds__(256) void gemm_tile_kernel(const int8_t *__restrict__ xq, const float *__restrict__ s_tok,
                                                        const uint8_t *__restrict__ wq, const float *__restrict__ s_w,
                                                        int gs, const half_t *__restrict__ bias, int M, int N, int K,
                                                        half_t *__restrict__ out, int32_t *__restrict__ acc_out,
                                                        int tiles_m, int tiles_n) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int BK = 128;
    constexpr int X_STAGE = BM * BK;
    constexpr int W_STAGE = BN * BK;
    constexpr int STAGE = X_STAGE + W_STAGE;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int XU = BM / 8;                       // 1 KB load units (8 rows) in the activation tile
    constexpr int WU = BN / 8;
    constexpr int DIRECT_UNITS = (WBITS == 8) ? (XU + WU) : XU;
    constexpr int LPS = DIRECT_UNITS / 4;            // direct loads per wave per stage
    constexpr int W4_PASSES = BN / 64;               // INT4: 4 threads per row, 64 rows per pass

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);

    // ---- tile coordinates, XCD aware --------------------------------------
    const int nb = tiles_m * tiles_n;
    const int b = blockIdx.x;
    const int xcd = b % 8;
    const int per = nb / 8, rem = nb % 8;
    const int t = xcd * per + (xcd < rem ? xcd : rem) + b / 8;   // XCD x owns a contiguous run of logical tiles
    constexpr int GM = 8;                                        // tile rows per band
    const int band = t / (GM * tiles_n);
    const int band_rows = (tiles_m - band * GM) < GM ? (tiles_m - band * GM) : GM;
    const int within = t - band * GM * tiles_n;
    const int tm = band * GM + within % band_rows;
    const int tn = within / band_rows;
    const int m0 = tm * BM;
    const int n0 = tn * BN;

    const int wrow_bytes = (WBITS == 8) ? K : K / 2;
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(wq), 0, (int)((size_t)N * wrow_bytes), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(xq), 0, (int)((size_t)M * K), kRsrcFlags);

    // ---- per-lane source offsets of this wave's direct-load units ---------
    // unit u < XU: activation rows u*8..u*8+7; else weight rows.  Rows past the
    // matrix edge are clamped to the last row: loaded, multiplied, never stored.
    int voff[LPS];
#pragma unroll
    for (int i = 0; i < LPS; ++i) {
        const int u = wave + 4 * i;
        if (u < XU) {
            const int row = u * 8 + lane / 8;
            int grow = m0 + row;
            if (grow > M - 1) grow = M - 1;
            voff[i] = grow * K + (((lane % 8) ^ swz(row)) * 16);
        } else {
            const int row = (u - XU) * 8 + lane / 8;
            int grow = n0 + row;
            if (grow > N - 1) grow = N - 1;
            voff[i] = grow * wrow_bytes + (((lane % 8) ^ swz(row)) * 16);
        }
    }
    // INT4 weights: thread -> (row = pass*64 + tid/4, 16 packed bytes = 32 codes = chunks 2q, 2q+1)
    int w4_voff[W4_PASSES > 0 ? W4_PASSES : 1];
    if (WBITS == 4) {
#pragma unroll
        for (int p = 0; p < W4_PASSES; ++p) {
            int grow = n0 + p * 64 + (int)threadIdx.x / 4;
            if (grow > N - 1) grow = N - 1;
            w4_voff[p] = grow * wrow_bytes + ((int)threadIdx.x % 4) * 16;
        }
    }

    auto issue_direct = [&](int kt, int slot) {
        uint8_t *base = smem + slot * STAGE;
#pragma unroll
        for (int i = 0; i < LPS; ++i) {
            const int u = wave + 4 * i;
            if (u < XU)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(base + u * 1024), 16, voff[i], kt * BK, 0,
                                                         0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, (lds_void *)(base + X_STAGE + (u - XU) * 1024), 16,
                                                         voff[i], kt * BK, 0, 0);
        }
    };
    int32x4 w4_regs[W4_PASSES > 0 ? W4_PASSES : 1];
    auto w4_fetch = [&](int kt) {
#pragma unroll
        for (int p = 0; p < W4_PASSES; ++p)
            w4_regs[p] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, w4_voff[p], kt * (BK / 2), 0);
    };
    auto w4_store = [&](int slot) {
        uint8_t *base = smem + slot * STAGE + X_STAGE;
#pragma unroll
        for (int p = 0; p < W4_PASSES; ++p) {
            const int row = p * 64 + (int)threadIdx.x / 4;
            const int q = (int)threadIdx.x % 4;
            uint32_t d[8];
            unpack8_nat((uint32_t)w4_regs[p][0], d[0], d[1]);
            unpack8_nat((uint32_t)w4_regs[p][1], d[2], d[3]);
            unpack8_nat((uint32_t)w4_regs[p][2], d[4], d[5]);
            unpack8_nat((uint32_t)w4_regs[p][3], d[6], d[7]);
            const int s = swz(row);
            *reinterpret_cast<int32x4 *>(base + row * BK + (((2 * q) ^ s) * 16)) =
                int32x4{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
            *reinterpret_cast<int32x4 *>(base + row * BK + (((2 * q + 1) ^ s) * 16)) =
                int32x4{(int)d[4], (int)d[5], (int)d[6], (int)d[7]};
        }
    };

    // ---- accumulators -----------------------------------------------------
    int32x16 acc[FN][FM];
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[fn][fm][e] = 0;

    const int wm = wave % 2, wn = wave / 2;
    const int lr = lane % 32;                // fragment row supplied by this lane
    const int lc = lane / 32;                // which 16-byte half of the 32-byte k step
    const int sw = swz(lr);                  // wave and fragment offsets are multiples of 32 rows
    const int x_off = (wm * WM + lr) * BK;
    const int w_off = X_STAGE + (wn * WN + lr) * BK;

    const int nkt = K / BK;
    issue_direct(0, 0);
    if (WBITS == 4) {
        w4_fetch(0);
        w4_store(0);
    }
    for (int kt = 0; kt < nkt; ++kt) {
        wait_vmcnt<0>();                     // this wave's loads of stage kt have landed
        __syncthreads();                     // ... and everyone's; stage kt-1 is no longer being read
        const int nxt = (kt + 1) & 1;
        if (kt + 1 < nkt) {
            issue_direct(kt + 1, nxt);
            if (WBITS == 4) w4_fetch(kt + 1);
        }
        const uint8_t *sb = smem + (kt & 1) * STAGE;
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            const int p = ((ks * 2 + lc) ^ sw) * 16;
            int32x4 a[FN], bx[FM];
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) a[fn] = *reinterpret_cast<const int32x4 *>(sb + w_off + fn * 32 * BK + p);
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) bx[fm] = *reinterpret_cast<const int32x4 *>(sb + x_off + fm * 32 * BK + p);
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
                    acc[fn][fm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[fn], bx[fm], acc[fn][fm], 0, 0, 0);
        }
        if (WBITS == 4 && kt + 1 < nkt) w4_store(nxt);   // slot nxt was last read before this iteration's barrier
    }

    // ---- epilogue ---------------------------------------------------------
    // acc[fn][fm][v]: output column n = wn*WN + fn*32 + 8*(v/4) + 4*(lane/32) + v%4,
    //                 token row     m = wm*WM + fm*32 + lane%32.
    __syncthreads();                          // all reads of the last stage are done; LDS is reused below
    constexpr int OROW = WN * 2 + 16;         // padded row of the wave's FP16 tile in LDS
    // (the launcher sizes dynamic LDS as max(2 * STAGE, 4 * WM * OROW))
    uint8_t *ot = smem + wave * (WM * OROW);
    const int mw = m0 + wm * WM;              // first token row of this wave
    const int nw = n0 + wn * WN;              // first output column of this wave
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
        const int m = mw + fm * 32 + lr;
        const float st = s_tok[m < M ? m : M - 1];
#pragma unroll
        for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int nl = fn * 32 + 8 * q + 4 * lc;
                int n = nw + nl;
                if (n > N - 4) n = N - 4;     // columns past N are never stored; keep the loads in range
                const float sc = st * s_w[n / gs];
                int32x4 v = {acc[fn][fm][4 * q], acc[fn][fm][4 * q + 1], acc[fn][fm][4 * q + 2],
                             acc[fn][fm][4 * q + 3]};
                if (WBITS == 4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] >>= 4;
                }
                half4 o;
                if (bias != nullptr) {
                    const half4 bv = *reinterpret_cast<const half4 *>(bias + n);
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (half_t)((float)v[e] * sc + (float)bv[e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (half_t)((float)v[e] * sc);
                }
                *reinterpret_cast<half4 *>(ot + (fm * 32 + lr) * OROW + nl * 2) = o;
                if (acc_out != nullptr && m < M && nw + nl < N)
                    *reinterpret_cast<int32x4 *>(acc_out + (size_t)m * N + nw + nl) = v;
            }
        }
    }
    // Each wave reads back its own tile only: a wave-local exchange, no workgroup barrier needed,
    // but the LDS writes above must have completed.
    __builtin_amdgcn_s_waitcnt(0xc07f);       // lgkmcnt(0)
    constexpr int LPR = WN * 2 / 16;          // lanes per output row (16 bytes each)
    constexpr int RPI = 64 / LPR;             // rows per store instruction
#pragma unroll
    for (int i = 0; i < WM / RPI; ++i) {
        const int row = i * RPI + lane / LPR;
        const int col = (lane % LPR) * 8;
        const int32x4 v = *reinterpret_cast<const int32x4 *>(ot + row * OROW + col * 2);
        const int m = mw + row;
        const int n = nw + col;
        if (m < M && n < N) *reinterpret_cast<int32x4 *>(out + (size_t)m * N + n) = v;
    }
#endif
}

namespace {

template <int BM, int BN, int WBITS>
hipError_t launch_tile_t(const GemmArgs &a, hipStream_t st) {
    constexpr int STAGE = (BM + BN) * 128;
    constexpr int OROW = BN + 16;
    constexpr size_t lds_main = 2 * STAGE;
    constexpr size_t lds_epi = 4 * (BM / 2) * OROW;
    constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_tile_kernel<BM, BN, WBITS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WBITS>), dim3(tiles_m * tiles_n), dim3(256), lds, st, a.xq, a.s_tok,
                       reinterpret_cast<const uint8_t *>(a.wq), a.s_w, a.N / a.groups,
                       reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K, reinterpret_cast<half_t *>(a.out),
                       a.acc_out, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_tile(const GemmArgs &a, int block, hipStream_t st) {
    if (block == 256) {
        if (a.w_bits == 8) return launch_tile_t<256, 256, 8>(a, st);
        return launch_tile_t<256, 256, 4>(a, st);
    }
    if (a.w_bits == 8) return launch_tile_t<128, 128, 8>(a, st);
    return launch_tile_t<128, 128, 4>(a, st);
}

}  // namespace zq
