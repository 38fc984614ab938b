// Weight-streaming GeMM for small token counts (M <= 64), with the
// dequantization epilogue (Sec. 4.3: at small batch the latency is the time to
// load the weights from memory; App. D: the schedule is chosen from
// batch x sequence length).
//
// The kernel is bound by HBM: every weight byte is read once, with fully
// coalesced 16-byte direct-to-LDS loads (8 rows x 128 B per wave instruction)
// kept several stages ahead of the consumer, so a workgroup always has tens of
// KB in flight.  A workgroup owns 64 weight rows (one 16-row strip per wave)
// and a slice of K; the activation tile of that slice is staged once in LDS
// and shared by the four waves.  The product runs on v_mfma_i32_16x16x64_i8
// with the weight strip as the first operand, which leaves four consecutive
// output columns in each lane's accumulator.  INT4 weights are unpacked in
// registers: (p << 4) & 0xF0F0F0F0 and p & 0xF0F0F0F0 are the even and odd
// nibbles as int8 values scaled by 16; the activation bytes are permuted the
// same way and the exact factor 16 is shifted out of the accumulator.
//
// When N/64 alone gives too few workgroups, K is split across workgroups:
// INT32 partial sums go to the caller's workspace and a second kernel adds
// them in a fixed order and applies the epilogue (integer addition, so the
// result does not depend on timing).
#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

namespace {

constexpr uint32_t kRsrcFlags = 0x00020000u;   // raw 32-bit buffer, gfx9 encoding

typedef __attribute__((address_space(3))) void lds_void;

// 16-byte chunk position of chunk c in a row: rows r..r+15 land in 16
// different bank groups for any fixed c.
__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ void unpack_w4(uint2 p, int32x4 &a) {
    a[0] = (int)((p.x << 4) & 0xf0f0f0f0u);   // k 0,2,4,6   (x16)
    a[1] = (int)(p.x & 0xf0f0f0f0u);          // k 1,3,5,7
    a[2] = (int)((p.y << 4) & 0xf0f0f0f0u);   // k 8,10,12,14
    a[3] = (int)(p.y & 0xf0f0f0f0u);          // k 9,11,13,15
}

__device__ __forceinline__ void permute_x4(int32x4 x, int32x4 &b) {
    // gather even / odd bytes of each 8-byte half, matching unpack_w4
    b[0] = (int)__builtin_amdgcn_perm((uint32_t)x[1], (uint32_t)x[0], 0x06040200u);
    b[1] = (int)__builtin_amdgcn_perm((uint32_t)x[1], (uint32_t)x[0], 0x07050301u);
    b[2] = (int)__builtin_amdgcn_perm((uint32_t)x[3], (uint32_t)x[2], 0x06040200u);
    b[3] = (int)__builtin_amdgcn_perm((uint32_t)x[3], (uint32_t)x[2], 0x07050301u);
}

}  // namespace

template <int MT, int WBITS, int NSTAGE>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const int8_t *__restrict__ xq,
                                                          const float *__restrict__ s_tok,
                                                          const uint8_t *__restrict__ wq,
                                                          const float *__restrict__ s_w, int gs,
                                                          const half_t *__restrict__ bias, int M, int N, int K,
                                                          half_t *__restrict__ out, int32_t *__restrict__ acc_out,
                                                          int32_t *__restrict__ partial, int stages_per_split) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int KS = (WBITS == 8) ? 128 : 256;      // k elements per stage
    constexpr int W_STAGE = 64 * 128;                 // 64 rows x 128 bytes (packed bytes for INT4)
    constexpr int X_STAGE = MT * 16 * KS;
    constexpr int STAGE = W_STAGE + X_STAGE;
    constexpr int CPR = KS / 16;                      // 16-byte chunks per activation row
    constexpr int RPU = 64 / CPR;                     // activation rows per 1 KB load unit
    constexpr int UNITS = 8 + X_STAGE / 1024;         // 1 KB load units per stage
    constexpr int LPS = (UNITS + 3) / 4;              // loads per wave per stage
    constexpr int KSTEPS = KS / 64;

    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int r = lane % 16;
    const int j = lane / 16;
    const int n0 = blockIdx.x * 64;
    const int wrow_bytes = (WBITS == 8) ? K : K / 2;
    const int total_stages = K / KS;
    const int st_lo = blockIdx.y * stages_per_split;
    int st_hi = st_lo + stages_per_split;
    if (st_hi > total_stages) st_hi = total_stages;
    const int nst = st_hi - st_lo;

    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(wq), 0, (int)((size_t)N * wrow_bytes), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(xq), 0, (int)((size_t)M * K), kRsrcFlags);

    // Per-lane source offsets of this wave's load units (wave w takes units w, w+4, ...;
    // a wrapped index repeats a unit with identical data, keeping the per-wave load count uniform).
    int voff[LPS];
    int ldso[LPS];
    bool is_w[LPS];
#pragma unroll
    for (int i = 0; i < LPS; ++i) {
        const int u = (wave + 4 * i) % UNITS;
        is_w[i] = u < 8;
        if (u < 8) {
            const int row = u * 8 + lane / 8;
            int grow = n0 + row;
            if (grow > N - 1) grow = N - 1;
            voff[i] = grow * wrow_bytes + (((lane % 8) ^ swz(row)) * 16);
            ldso[i] = u * 1024;
        } else {
            const int ux = u - 8;
            const int row = ux * RPU + lane / CPR;
            int grow = row;
            if (grow > M - 1) grow = M - 1;
            voff[i] = grow * K + (((lane % CPR) ^ swz(row)) * 16);
            ldso[i] = W_STAGE + ux * 1024;
        }
    }

    auto issue = [&](int stage_abs, int slot) {
        uint8_t *base = smem + slot * STAGE;
#pragma unroll
        for (int i = 0; i < LPS; ++i) {
            if (is_w[i])
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, (lds_void *)(base + ldso[i]), 16, voff[i],
                                                         stage_abs * 128, 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(base + ldso[i]), 16, voff[i],
                                                         stage_abs * KS, 0, 0);
        }
    };

    const int sw = swz(r);
    const int wrow_off = (wave * 16 + r) * 128;

    int32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = int32x4{0, 0, 0, 0};

#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < nst) issue(st_lo + s, s);

    for (int kt = 0; kt < nst; ++kt) {
        // Stage kt has landed once at most the loads of the NSTAGE-2 later stages are outstanding.
        if (kt + NSTAGE - 2 < nst)
            wait_vmcnt<(NSTAGE - 2) * LPS>();
        else
            wait_vmcnt<0>();
        __syncthreads();
        if (kt + NSTAGE - 1 < nst) issue(st_lo + kt + NSTAGE - 1, (kt + NSTAGE - 1) % NSTAGE);
        const uint8_t *sb = smem + (kt % NSTAGE) * STAGE;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int c = ks * 4 + j;                 // 16-byte chunk of activations for this lane
            int32x4 a;
            if (WBITS == 8) {
                a = *reinterpret_cast<const int32x4 *>(sb + wrow_off + ((c ^ sw) * 16));
            } else {
                const int cw = ks * 2 + (j >> 1);     // packed chunk; this lane's 8 bytes are its half
                const uint2 p = *reinterpret_cast<const uint2 *>(sb + wrow_off + ((cw ^ sw) * 16) + (j & 1) * 8);
                unpack_w4(p, a);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                int32x4 b = *reinterpret_cast<const int32x4 *>(sb + W_STAGE + (mt * 16 + r) * KS + ((c ^ sw) * 16));
                if (WBITS == 4) {
                    int32x4 bp;
                    permute_x4(b, bp);
                    b = bp;
                }
                acc[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[mt], 0, 0, 0);
            }
        }
    }

    const int nrow = n0 + wave * 16;
    if (nrow >= N) return;
    const int n = nrow + 4 * j;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + r;
        if (m >= M) continue;
        int32x4 v = acc[mt];
        if (WBITS == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] >>= 4;   // exact: every product carried the factor 16
        }
        if (partial != nullptr) {
            *reinterpret_cast<int32x4 *>(partial + ((size_t)blockIdx.y * M + m) * N + n) = v;
        } else {
            const float sc = s_tok[m] * s_w[n / gs];
            half4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float f = (float)v[e] * sc;
                if (bias != nullptr) f += (float)bias[n + e];
                o[e] = (half_t)f;
            }
            *reinterpret_cast<half4 *>(out + (size_t)m * N + n) = o;
            if (acc_out != nullptr) *reinterpret_cast<int32x4 *>(acc_out + (size_t)m * N + n) = v;
        }
    }
#endif
}

// Sum the split-K partials in split order and apply the epilogue; one thread per four columns.
__global__ __launch_bounds__(256) void splitk_epilogue_kernel(const int32_t *__restrict__ partial, int splits,
                                                              const float *__restrict__ s_tok,
                                                              const float *__restrict__ s_w, int gs,
                                                              const half_t *__restrict__ bias, int M, int N,
                                                              half_t *__restrict__ out, int32_t *__restrict__ acc_out) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const long quads = (long)M * (N / 4);
    if (idx >= quads) return;
    const int m = (int)(idx / (N / 4));
    const int n = (int)(idx % (N / 4)) * 4;
    int32x4 v = {0, 0, 0, 0};
    for (int s = 0; s < splits; ++s)
        v += *reinterpret_cast<const int32x4 *>(partial + ((size_t)s * M + m) * N + n);
    const float sc = s_tok[m] * s_w[n / gs];
    half4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float f = (float)v[e] * sc;
        if (bias != nullptr) f += (float)bias[n + e];
        o[e] = (half_t)f;
    }
    *reinterpret_cast<half4 *>(out + (size_t)m * N + n) = o;
    if (acc_out != nullptr) *reinterpret_cast<int32x4 *>(acc_out + (size_t)m * N + n) = v;
}

namespace {

constexpr int kSkinnyStages = 4;

template <int MT, int WBITS>
hipError_t launch_skinny_t(const GemmArgs &a, int splits, int stages_per_split, hipStream_t st) {
    constexpr int KS = (WBITS == 8) ? 128 : 256;
    constexpr int STAGE = 64 * 128 + MT * 16 * KS;
    const size_t lds = (size_t)kSkinnyStages * STAGE;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void *>(&gemm_skinny_kernel<MT, WBITS, kSkinnyStages>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid((a.N + 63) / 64, splits);
    int32_t *partial = splits > 1 ? reinterpret_cast<int32_t *>(a.workspace) : nullptr;
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, WBITS, kSkinnyStages>), grid, dim3(256), lds, st, a.xq, a.s_tok, reinterpret_cast<const uint8_t *>(a.wq), a.s_w,
                       a.N / a.groups, reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K,
                       reinterpret_cast<half_t *>(a.out), a.acc_out, partial, stages_per_split);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (splits > 1) {
        const long quads = (long)a.M * (a.N / 4);
        hipLaunchKernelGGL(splitk_epilogue_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, partial,
                           splits, a.s_tok, a.s_w, a.N / a.groups, reinterpret_cast<const half_t *>(a.bias), a.M, a.N,
                           reinterpret_cast<half_t *>(a.out), a.acc_out);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace

// Number of K splits for the skinny schedule: enough workgroups to keep every
// CU streaming (about three per CU), never fewer than four stages per split.
int skinny_splits(int N, int K, int w_bits) {
    const int ks = (w_bits == 8) ? 128 : 256;
    const int stages = K / ks;
    const int tiles = (N + 63) / 64;
    int s = (768 + tiles / 2) / tiles;
    if (s > stages / 4) s = stages / 4;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return s;
}

hipError_t launch_gemm_skinny(const GemmArgs &a, bool split_k, hipStream_t st) {
    const int ks = (a.w_bits == 8) ? 128 : 256;
    const int stages = a.K / ks;
    int splits = split_k ? skinny_splits(a.N, a.K, a.w_bits) : 1;
    int sps = (stages + splits - 1) / splits;
    splits = (stages + sps - 1) / sps;            // no empty split
    const int mt = (a.M + 15) / 16;
#define ZQ_SK(MT, WB) return launch_skinny_t<MT, WB>(a, splits, sps, st)
    if (a.w_bits == 8) {
        if (mt <= 1) ZQ_SK(1, 8);
        if (mt <= 2) ZQ_SK(2, 8);
        ZQ_SK(4, 8);
    } else {
        if (mt <= 1) ZQ_SK(1, 4);
        if (mt <= 2) ZQ_SK(2, 4);
        ZQ_SK(4, 4);
    }
#undef ZQ_SK
}

}  // namespace zq
