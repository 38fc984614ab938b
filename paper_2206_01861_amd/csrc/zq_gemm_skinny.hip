// Weight-streaming GeMM for small token counts (M <= 64), with the
// dequantization epilogue (Sec. 4.3: at small batch the latency is the time to
// load the weights from memory; App. D: the schedule is chosen from
// batch x sequence length).
//
// The kernel is bound by HBM, so it is built around bytes in flight.  A
// workgroup has four consumer waves and one producer wave and owns 64 weight
// rows (one 16-row strip per consumer) over a slice of K, in stages of 256
// values of K:
//   * each consumer streams its own strip straight into registers, DW stages
//     ahead (16-byte buffer loads; the four loads of a stage cover 256
//     contiguous bytes of each row).  Registers hold far more outstanding
//     bytes than LDS could, and a consumer waits only on its own loads;
//   * the producer wave copies the activation tile of each stage from L2 into
//     an LDS ring with 16-byte direct-to-LDS loads, R-1 stages ahead; its load
//     counter is separate from the consumers', so a slow HBM load never holds
//     back the activations and vice versa.  One workgroup barrier per stage
//     hands a filled slot to the consumers and a drained slot back.
// The product runs on v_mfma_i32_16x16x64_i8 with the weight strip as the
// first operand, which leaves four consecutive output columns in each lane's
// accumulator.  INT4 weights are unpacked in registers: (p << 4) & 0xF0F0F0F0
// and p & 0xF0F0F0F0 are the even and odd nibbles as int8 values scaled by 16;
// the activation bytes are permuted the same way and the exact factor 16 is
// shifted out of the accumulator.
//
// When N/64 alone gives too few workgroups, K is split across workgroups:
// INT32 partial sums go to the caller's workspace and the workgroup that
// finishes a tile last adds them in split order and applies the epilogue
// (integer addition, so the result does not depend on timing).
#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

namespace {

constexpr uint32_t kRsrcFlags = 0x00020000u;   // raw 32-bit buffer, gfx9 encoding
constexpr int kMaxSplitTiles = 8192;
constexpr int kStageK = 256;                   // values of K per stage
constexpr int kAuxDeviceCoherent = 0x10;        // sc1: coherent across the XCDs of the device
constexpr int kStreamDepth = 4;                // weight stages a consumer keeps in flight

typedef __attribute__((address_space(3))) void lds_void;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ int32x4 unpack_w4(uint32_t p0, uint32_t p1) {
    int32x4 a;
    a[0] = (int)((p0 << 4) & 0xf0f0f0f0u);   // k 0,2,4,6   (x16)
    a[1] = (int)(p0 & 0xf0f0f0f0u);          // k 1,3,5,7
    a[2] = (int)((p1 << 4) & 0xf0f0f0f0u);   // k 8,10,12,14
    a[3] = (int)(p1 & 0xf0f0f0f0u);          // k 9,11,13,15
    return a;
}

__device__ __forceinline__ int32x4 permute_x4(int32x4 x) {
    // gather even / odd bytes of each 8-byte half, matching unpack_w4
    int32x4 b;
    b[0] = (int)__builtin_amdgcn_perm((uint32_t)x[1], (uint32_t)x[0], 0x06040200u);
    b[1] = (int)__builtin_amdgcn_perm((uint32_t)x[1], (uint32_t)x[0], 0x07050301u);
    b[2] = (int)__builtin_amdgcn_perm((uint32_t)x[3], (uint32_t)x[2], 0x06040200u);
    b[3] = (int)__builtin_amdgcn_perm((uint32_t)x[3], (uint32_t)x[2], 0x07050301u);
    return b;
}

// The weight stream is issued and awaited with explicit instructions.  The compiler's automatic
// wait insertion cannot count loads that stay in flight across a loop back-edge and falls back
// to draining the whole queue (vmcnt(0)) at every use, which would leave one stage in flight
// instead of DW.  A load written as an asm statement is not tracked by the compiler; the
// matching wait names the destination registers as in/out operands, so no use of the data can
// be scheduled above it.
typedef uint32_t uint32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32x4 make_srd(const void *p, uint32_t bytes) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    uint32x4 d;
    d[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
    d[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
    d[2] = __builtin_amdgcn_readfirstlane(bytes);    // bounds: reads past the matrix return 0, never fault
    d[3] = kRsrcFlags;
    return d;
}

template <int IMM>
__device__ __forceinline__ void stream_load16(int32x4 &dst, int voff, uint32x4 srd, int soff) {
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen offset:%4"
                 : "=&v"(dst)
                 : "v"(voff), "s"(srd), "s"(soff), "n"(IMM));
}

template <int N, int LW>
__device__ __forceinline__ void stream_wait(int32x4 (&w)[LW]) {
    if (LW == 4)
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]) : "n"(N));
    else
        asm volatile("s_waitcnt vmcnt(%2)" : "+v"(w[0]), "+v"(w[1]) : "n"(N));
}

}  // namespace

// Arrival counters of the split-K tiles.  Zero when the library is loaded and zero again after
// every call (the last workgroup of a tile resets its counter), so no launch is spent clearing
// them.  Shared by all calls on a device: split-K GeMM calls must not overlap on one device.
__device__ unsigned int g_tile_arrivals[kMaxSplitTiles];

template <int MT, int WBITS, int DW, int R>
__global__ __launch_bounds__(320) void gemm_stream_kernel(const int8_t *__restrict__ xq,
                                                          const float *__restrict__ s_tok,
                                                          const uint8_t *__restrict__ wq,
                                                          const float *__restrict__ s_w, int gs,
                                                          const half_t *__restrict__ bias, int M, int N, int K,
                                                          half_t *__restrict__ out, int32_t *__restrict__ acc_out,
                                                          int32_t *__restrict__ partial, int stages_per_split) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int LW = (WBITS == 8) ? 4 : 2;          // 16-byte weight loads per lane per stage
    constexpr int X_STAGE = MT * 16 * kStageK;        // bytes of one activation stage
    constexpr int LX = X_STAGE / 1024;                // 1 KB direct loads per stage (producer wave)

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r = lane % 16;
    const int j = lane / 16;
    const int n0 = blockIdx.x * 64;
    const int total_stages = K / kStageK;
    const int st_lo = blockIdx.y * stages_per_split;
    int st_hi = st_lo + stages_per_split;
    if (st_hi > total_stages) st_hi = total_stages;
    const int nst = st_hi - st_lo;

    if (wave == 4) {
        // ---- producer: activation stages into the LDS ring ------------------
        // A 1 KB unit is 4 rows x 256 bytes; chunk c of row m sits at position c ^ (m & 15),
        // which makes the consumers' fragment reads (16 rows, one chunk) conflict free.
        const __amdgpu_buffer_rsrc_t rs_x =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(xq), 0, (int)((size_t)M * K), kRsrcFlags);
        int voff[LX];
#pragma unroll
        for (int u = 0; u < LX; ++u) {
            const int row = u * 4 + lane / 16;
            int grow = row;
            if (grow > M - 1) grow = M - 1;           // rows past M: valid data, results never stored
            voff[u] = grow * K + (((lane % 16) ^ (row & 15)) * 16);
        }
        auto issue_x = [&](int stage_abs, int slot) {
            uint8_t *base = smem + slot * X_STAGE;
#pragma unroll
            for (int u = 0; u < LX; ++u)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(base + u * 1024), 16, voff[u],
                                                         stage_abs * kStageK, 0, 0);
        };
#pragma unroll
        for (int s = 0; s < R - 1; ++s)
            if (s < nst) issue_x(st_lo + s, s);
        for (int kt = 0; kt < nst; ++kt) {
            // Stage kt has landed once at most the R-2 later stages are outstanding.
            if (kt + R - 2 < nst)
                wait_vmcnt<(R - 2) * LX>();
            else
                wait_vmcnt<0>();
            lds_barrier();                            // slot kt filled; slot kt-1 drained by every consumer
            if (kt + R - 1 < nst) issue_x(st_lo + kt + R - 1, (kt + R - 1) % R);
        }
        if (gridDim.y > 1) {                          // keep the two barriers of the split-K hand-over balanced
            lds_barrier();
            __syncthreads();
        }
        return;
    }

    // ---- consumers: weight strip through registers ------------------------
    const int wrow_bytes = (WBITS == 8) ? K : K / 2;
    const uint32x4 rs_w = make_srd(wq, (uint32_t)((size_t)N * wrow_bytes));
    int wrow = n0 + wave * 16 + r;
    if (wrow > N - 1) wrow = N - 1;
    const int voff_w = wrow * wrow_bytes + j * 16;
    constexpr int W_STAGE_BYTES = (WBITS == 8) ? kStageK : kStageK / 2;   // bytes of a row per stage

    int32x4 wreg[DW][LW];
    auto issue_w = [&](int stage_abs, int32x4(&dst)[LW]) {
        const int soff = stage_abs * W_STAGE_BYTES;
        stream_load16<0>(dst[0], voff_w, rs_w, soff);
        stream_load16<64>(dst[1], voff_w, rs_w, soff);
        if (LW == 4) {
            stream_load16<128>(dst[2], voff_w, rs_w, soff);
            stream_load16<192>(dst[3], voff_w, rs_w, soff);
        }
    };

    int32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = int32x4{0, 0, 0, 0};

    const int x_lane = r * kStageK;                   // this lane's row inside a 16-row block
    auto compute = [&](const int32x4(&w)[LW], const uint8_t *xs) {
        if (WBITS == 8) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {             // k step i: bytes 64i + 16j of the stage
                const int c = 4 * i + j;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int32x4 b =
                        *reinterpret_cast<const int32x4 *>(xs + mt * 16 * kStageK + x_lane + ((c ^ r) * 16));
                    acc[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w[i], b, acc[mt], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i) {             // 16 packed bytes = codes 128i + 32j .. +31
#pragma unroll
                for (int h = 0; h < 2; ++h) {         // two k steps of 16 codes each
                    const int32x4 a = unpack_w4((uint32_t)w[i][2 * h], (uint32_t)w[i][2 * h + 1]);
                    const int c = 8 * i + 2 * j + h;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const int32x4 b =
                            *reinterpret_cast<const int32x4 *>(xs + mt * 16 * kStageK + x_lane + ((c ^ r) * 16));
                        acc[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, permute_x4(b), acc[mt], 0, 0, 0);
                    }
                }
            }
        }
    };

    // The slice is processed in groups of DW stages.  Everything on the streamed path is
    // unconditional, so a register that is the target of a load in flight is never copied or
    // merged by the compiler: issue group 0; for every further group, step through the stages,
    // each step waiting for its stage, computing it and refilling the register set it just freed
    // with the same stage of the next group; finally drain the last group.
    const int ngroups = nst / DW;
    int kt = 0;
    if (ngroups >= 1) {
#pragma unroll
        for (int d = 0; d < DW; ++d) issue_w(st_lo + d, wreg[d]);
        for (int g = 1; g < ngroups; ++g) {
#pragma unroll
            for (int d = 0; d < DW; ++d) {
                stream_wait<(DW - 1) * LW, LW>(wreg[d]);   // at most DW-1 later stages outstanding
                lds_barrier();                              // activation slot of stage kt is filled
                compute(wreg[d], smem + (kt % R) * X_STAGE);
                issue_w(st_lo + kt + DW, wreg[d]);
                ++kt;
            }
        }
        static_assert(DW == 4, "the drain below is written out for four stages");
#define ZQ_DRAIN(d)                                         \
    stream_wait<(DW - 1 - (d)) * LW, LW>(wreg[d]);         \
    lds_barrier();                                          \
    compute(wreg[d], smem + (kt % R) * X_STAGE);            \
    ++kt;
        ZQ_DRAIN(0)
        ZQ_DRAIN(1)
        ZQ_DRAIN(2)
        ZQ_DRAIN(3)
#undef ZQ_DRAIN
    }
    // Stages that do not fill a group (K/256 not a multiple of DW, or an uneven split): plain
    // loads, one stage at a time.
    for (; kt < nst; ++kt) {
        const __amdgpu_buffer_rsrc_t rs_plain = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t *>(wq), 0, (int)((size_t)N * wrow_bytes), kRsrcFlags);
        int32x4 w[LW];
#pragma unroll
        for (int i = 0; i < LW; ++i)
            w[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_plain, voff_w, (st_lo + kt) * W_STAGE_BYTES + i * 64, 0);
        lds_barrier();
        compute(w, smem + (kt % R) * X_STAGE);
    }

    // ---- epilogue ---------------------------------------------------------
    // One split: dequantize straight from the accumulators.  Several splits: every workgroup
    // parks its INT32 partial tile in the workspace and bumps the tile's arrival counter; the
    // workgroup that arrives last adds the partials in split order (integer sums: the result
    // does not depend on arrival order), dequantizes, and resets the counter for the next call.
    // The producer wave takes part in the two barriers of the hand-over and then leaves.
    if (WBITS == 4) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[mt][e] >>= 4;   // exact: every product carried the factor 16
    }
    const int nrow = n0 + wave * 16;
    const bool row_ok = nrow < N;
    const int n = nrow + 4 * j;
    const int splits = gridDim.y;
    if (splits > 1) {
        const __amdgpu_buffer_rsrc_t rs_p = __builtin_amdgcn_make_buffer_rsrc(
            partial, 0, (int)((size_t)splits * M * N * sizeof(int32_t)), kRsrcFlags);
        if (row_ok) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = mt * 16 + r;
                if (m < M) {
                    // 16-byte store with the device-coherence bit (sc1): written through, not left in this XCD's L2
                    __builtin_amdgcn_raw_buffer_store_b128(acc[mt], rs_p, (int)((((size_t)blockIdx.y * M + m) * N + n) * 4),
                                                           0, kAuxDeviceCoherent);
                }
            }
        }
        // The partials were written through to device-coherent memory; once every store of this
        // workgroup is acknowledged the arrival is counted.  No cache-wide fence is used: on a
        // multi-XCD part it would flush and invalidate the L2 that the other workgroups stream from.
        wait_vmcnt<0>();
        lds_barrier();
        __shared__ int is_last;
        if (threadIdx.x == 0) {
            const unsigned prev = __hip_atomic_fetch_add(&g_tile_arrivals[blockIdx.x], 1u, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == (unsigned)splits - 1u);
        }
        __syncthreads();
        if (!is_last) return;
        if (threadIdx.x == 0)
            __hip_atomic_store(&g_tile_arrivals[blockIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = int32x4{0, 0, 0, 0};
        if (row_ok) {
            for (int sp = 0; sp < splits; ++sp) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int m = mt * 16 + r;
                    if (m < M) {
                        acc[mt] += __builtin_amdgcn_raw_buffer_load_b128(
                            rs_p, (int)((((size_t)sp * M + m) * N + n) * 4), 0, kAuxDeviceCoherent);
                    }
                }
            }
        }
    }
    if (!row_ok) return;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + r;
        if (m >= M) continue;
        const int32x4 v = acc[mt];
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
#endif
}

namespace {

template <int MT, int WBITS>
hipError_t launch_stream_t(const GemmArgs &a, int splits, int stages_per_split, hipStream_t st) {
    constexpr int DW = kStreamDepth;
    constexpr int R = 3;
    constexpr size_t lds = (size_t)R * MT * 16 * kStageK;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_stream_kernel<MT, WBITS, DW, R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid((a.N + 63) / 64, splits);
    int32_t *partial = splits > 1 ? reinterpret_cast<int32_t *>(a.workspace) : nullptr;
    hipLaunchKernelGGL((gemm_stream_kernel<MT, WBITS, DW, R>), grid, dim3(320), lds, st, a.xq, a.s_tok,
                       reinterpret_cast<const uint8_t *>(a.wq), a.s_w, a.N / a.groups,
                       reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K, reinterpret_cast<half_t *>(a.out),
                       a.acc_out, partial, stages_per_split);
    return hipGetLastError();
}

}  // namespace

// Number of K splits for the streaming schedule: about one and a half workgroups per CU (more
// splits cost a round trip of INT32 partials for nothing), never fewer than four stages per split.
int skinny_splits(int N, int K, int w_bits) {
    (void)w_bits;
    const int stages = K / kStageK;
    const int tiles = (N + 63) / 64;
    if (tiles > kMaxSplitTiles) return 1;
    int s = (384 + tiles / 2) / tiles;
    if (s > stages / 4) s = stages / 4;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    while (s > 1 && (size_t)s * 64 * (size_t)N * sizeof(int32_t) >= ((size_t)1 << 31)) --s;   // 32-bit offsets
    return s;
}

hipError_t launch_gemm_skinny(const GemmArgs &a, bool split_k, hipStream_t st) {
    const int stages = a.K / kStageK;
    int splits = split_k ? skinny_splits(a.N, a.K, a.w_bits) : 1;
    int sps = (stages + splits - 1) / splits;
    if (splits > 1) sps = (sps + kStreamDepth - 1) / kStreamDepth * kStreamDepth;   // whole groups per split
    splits = (stages + sps - 1) / sps;            // no empty split
    const int mt = (a.M + 15) / 16;
#define ZQ_SK(MT, WB) return launch_stream_t<MT, WB>(a, splits, sps, st)
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
