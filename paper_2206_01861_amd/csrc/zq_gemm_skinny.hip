// Weight-streaming GeMM for small token counts (M <= 128), with the
// dequantization epilogue (Sec. 4.3: at small batch the latency is the time to
// load the weights from memory; App. D: the schedule is chosen from
// batch x sequence length).
//
// The kernel is bound by HBM, so it is built around bytes in flight.  A
// workgroup has one producer wave and up to eight consumer waves; each
// consumer owns one 16-row strip of the weight matrix over the workgroup's
// range of K, in stages of 256 values of K:
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
// Work is cut into row blocks x K splits.  A CU cannot pull more than its share
// of HBM bandwidth, so an idle or overloaded CU is lost time: the strips are
// dealt evenly over a number of row blocks that is a multiple of the CU count
// where N allows it (blocks differ by at most one strip; a wave without a strip
// only keeps the barriers), and only matrices with too few rows for that are
// also split along K.  The host picks the cut from a small cost model (bytes
// per CU, bytes in flight per CU, the fixed cost of the exchange).  With a K
// split every wave parks its INT32 partial strip in the caller's workspace with
// device-coherent 16-byte stores and counts its arrival with a relaxed atomic;
// the wave that arrives last adds the other partials and applies the epilogue
// (two's-complement addition: the result does not depend on timing).  The
// protocol is per wave and uses no barrier and no cache-wide fence (on a
// multi-XCD part a fence flushes and invalidates the L2 every workgroup streams
// from).
#include <type_traits>

#include "zq_device.h"
#include "zq_internal.h"

namespace zq {

namespace {

constexpr uint32_t kRsrcFlags = 0x00020000u;   // raw 32-bit buffer, gfx9 encoding
constexpr int kStageK = 256;                   // values of K per stage
[[maybe_unused]] constexpr int kAuxDeviceCoherent = 0x10;        // sc1: coherent across the XCDs of the device
constexpr int kMaxConsumers = 8;               // consumer waves per workgroup

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

// Weight loads of a 16-row strip, 64 bytes of each row per load.  The vector cache works through a
// load four lanes at a time and is fastest when those four lanes are contiguous in memory; in the
// matrix-core operand layout (lane = row a of 16, 16-byte chunk b of 4: consecutive lanes are
// consecutive rows) every group of four touches four lines, and that costs 12-15 % of the stream
// once the activation tile shares the cache (64 tokens).  So the loads run chunk-fastest (lane =
// 4a + b) and one cross-lane permutation per register turns the result into the operand layout.
template <int LW>
__device__ __forceinline__ void issue_strip(int32x4 (&dst)[LW], int voff, uint32x4 srd, int soff) {
    stream_load16<0>(dst[0], voff, srd, soff);
    stream_load16<64>(dst[1], voff, srd, soff);
    if (LW == 4) {
        stream_load16<128>(dst[2], voff, srd, soff);
        stream_load16<192>(dst[3], voff, srd, soff);
    }
}
// pull = 4 * (4 * (lane % 16) + lane / 16): byte address of the lane that holds (row lane%16, chunk lane/16).
template <int LW>
__device__ __forceinline__ void strip_operands(const int32x4 (&w)[LW], int32x4 (&t)[LW], int pull) {
#pragma unroll
    for (int i = 0; i < LW; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) t[i][e] = __builtin_amdgcn_ds_bpermute(pull, w[i][e]);
}

// One dword fetched the same way (used for the operands of the epilogue): issued here, not tracked
// by the compiler, usable only after a wait followed by landed().
__device__ __forceinline__ void async_load_dword(uint32_t &dst, const void *p) {
    asm volatile("global_load_dword %0, %1, off" : "=&v"(dst) : "v"(p));
}
// After a wait that covers it: from here on the register holds the loaded value.
__device__ __forceinline__ void landed(uint32_t &v) { asm volatile("" : "+v"(v)); }

template <int N, int LW>
__device__ __forceinline__ void stream_wait(int32x4 (&w)[LW]) {
    if (LW == 4)
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]) : "n"(N));
    else
        asm volatile("s_waitcnt vmcnt(%2)" : "+v"(w[0]), "+v"(w[1]) : "n"(N));
}

}  // namespace

// The arrival counters of the strips that are split along K live in the caller's workspace (one per
// strip, kMaxSharedStrips of them): zero after zq_workspace_init() and zero again after every call
// (the wave that completes a strip resets its counter), so no launch is spent clearing them.

struct StreamPlan {
    int strips;       // 16-row strips of the weight matrix (N / 16)
    int stages;       // stages of 256 K-values (K / 256)
    int row_blocks;   // workgroups along N; the strips are dealt out as evenly as whole strips allow
    int k_splits;     // workgroups along K; the stages likewise
    int consumers;    // consumer waves per workgroup = most strips in a row block
    // filled by finish_plan(): strips / row_blocks, strips % row_blocks, stages / k_splits, stages % k_splits
    int strips_per_block, strips_rem, stages_per_split, stages_rem;
    // 1: every strip of a row block is streamed by two waves, each over half of the block's K
    // range, and their accumulators are added through LDS at the end (see plan_stream)
    int range_shift = 0;
};

template <int MT, int WBITS, int DW, int R, int QSH = 0>
__global__ __launch_bounds__(64 * (kMaxConsumers + 1)) void gemm_stream_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ s_tok, const uint8_t *__restrict__ wq,
    const float *__restrict__ s_w, int gs, const half_t *__restrict__ bias, int M, int N, int K,
    half_t *__restrict__ out, int32_t *__restrict__ acc_out, int32_t *__restrict__ partial,
    unsigned *__restrict__ arrivals, StreamPlan plan, int act) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int LW = (WBITS == 8) ? 4 : 2;          // 16-byte weight loads per lane per stage
    constexpr int X_STAGE = MT * 16 * kStageK;        // bytes of one activation stage
    constexpr int LX = X_STAGE / 1024;                // 1 KB direct loads per stage (producer wave)

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r = lane % 16;
    const int j = lane / 16;

    // blockIdx.x = row block, blockIdx.y = K split; the first `rem` blocks of each kind take one more
    // strip / stage (the quotients come from the host: no integer division at the head of the kernel)
    const int rb = (int)blockIdx.x;
    const int ks = (int)blockIdx.y;
    const int s_lo = rb * plan.strips_per_block + (rb < plan.strips_rem ? rb : plan.strips_rem);
    const int s_hi = s_lo + plan.strips_per_block + (rb < plan.strips_rem ? 1 : 0);
    const int k_lo = ks * plan.stages_per_split + (ks < plan.stages_rem ? ks : plan.stages_rem);
    const int k_hi = k_lo + plan.stages_per_split + (ks < plan.stages_rem ? 1 : 0);
    const int n = k_hi - k_lo;                        // stages of this workgroup (>= 1: k_splits <= stages)
    constexpr int Q = 1 << QSH;                       // K ranges per strip (1, or 2 with QSH = 1)
    const int nq = (n + Q - 1) >> QSH;                // stages per range = steps of this workgroup
    const int npad = (nq + DW - 1) / DW * DW;         // the pipeline always runs whole groups of DW
    constexpr int SLOT = X_STAGE << QSH;              // a ring slot holds the activation stage of every range

    if (wave == 0) {
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
        // step i of range q is stage q*nq + i of this workgroup (past the end: the last stage again,
        // loaded and never multiplied)
        auto issue_x = [&](int i, int slot) __attribute__((always_inline)) {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                uint8_t *base = smem + slot * SLOT + q * X_STAGE;
                int stg = q * nq + i;
                if (Q > 1 && stg > n - 1) stg = n - 1;
                const int soff = (k_lo + stg) * kStageK;
#pragma unroll
                for (int u = 0; u < LX; ++u)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(base + u * 1024), 16, voff[u], soff, 0,
                                                             0);
            }
        };
        static_assert((R - 2) * LX * Q <= 63, "the wait count is a six-bit field");
#pragma unroll
        for (int s = 0; s < R - 1; ++s)
            if (s < nq) issue_x(s, s);
        for (int i = 0; i < npad; ++i) {
            if (i < nq) {
                // Step i has landed once at most the loads of the R-2 later steps are outstanding.
                if (i + R - 2 < nq)
                    wait_vmcnt<(R - 2) * LX * Q>();
                else
                    wait_vmcnt<0>();
            }
            lds_barrier();                            // slot i filled; slot i-1 drained by every consumer
            if (i + R - 1 < nq) issue_x(i + R - 1, (i + R - 1) % R);
        }
        return;
    }

    const int cidx = wave - 1;                        // consumer: (strip of the block, K range)
    const int q = cidx & (Q - 1);
    const int strip = s_lo + (cidx >> QSH);
    if (strip >= s_hi) {                              // no strip for this wave: keep the barrier count
        for (int i = 0; i < npad; ++i) lds_barrier();
        return;
    }
    int n_mine = n - q * nq;                          // stages of this wave's range
    n_mine = n_mine < 0 ? 0 : (n_mine > nq ? nq : n_mine);
    const int stg_last = n_mine > 0 ? q * nq + n_mine - 1 : n - 1;

    // ---- consumers: weight strip through registers ------------------------
    const int wrow_bytes = (WBITS == 8) ? K : K / 2;
    const uint32x4 rs_w = make_srd(wq, (uint32_t)((size_t)N * wrow_bytes));
    constexpr int W_STAGE_BYTES = (WBITS == 8) ? kStageK : kStageK / 2;   // bytes of a row per stage
    const int voff_w = (int)((uint32_t)(strip * 16 + lane / 4) * (uint32_t)wrow_bytes + (uint32_t)((lane % 4) * 16));
    const int pull = 4 * (4 * r + j);

    int32x4 wreg[DW][LW];
    // Stage i of this workgroup; indices past the end re-load the last stage (never computed).
    auto issue_w = [&](int i, int32x4(&dst)[LW]) __attribute__((always_inline)) {
        int stg = q * nq + i;
        if (stg > stg_last) stg = stg_last;
        const int soff = __builtin_amdgcn_readfirstlane((k_lo + stg) * W_STAGE_BYTES);   // wave-uniform by construction
        issue_strip<LW>(dst, voff_w, rs_w, soff);
    };

    int32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = int32x4{0, 0, 0, 0};

    const int x_lane = r * kStageK;                   // this lane's row inside a 16-row block
    auto compute = [&](const int32x4(&wl)[LW], const uint8_t *xs) __attribute__((always_inline)) {
        int32x4 w[LW];
        strip_operands<LW>(wl, w, pull);
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

    // The run is processed in groups of DW stages.  Everything that touches the streamed registers
    // is unconditional, so a register that is the target of a load in flight is never copied or
    // merged by the compiler: issue the first group; then step through the stages, each step
    // waiting for its stage, computing it (if it exists) and refilling the register set it just
    // freed with the stage DW further on; the last group only drains.
    int i = 0;
    auto step_compute = [&](const int32x4(&w)[LW]) __attribute__((always_inline)) {
        if (i < n_mine) compute(w, smem + (i % R) * SLOT + q * X_STAGE);
    };
#pragma unroll
    for (int d = 0; d < DW; ++d) issue_w(d, wreg[d]);
    for (int grp = DW; grp < npad; grp += DW) {
#pragma unroll
        for (int d = 0; d < DW; ++d) {
            stream_wait<(DW - 1) * LW, LW>(wreg[d]);   // at most DW-1 later stages outstanding
            lds_barrier();                              // activation slot of stage i is filled
            step_compute(wreg[d]);
            issue_w(i + DW, wreg[d]);
            ++i;
        }
    }
    // The operands of the epilogue are fetched now, under the last stages of the stream; otherwise
    // their L2 round trip would sit between the last MFMA and the first store.  Being younger than
    // every weight load still in flight they only make the waits of the drain a little stricter
    // than needed; the last of those waits (vmcnt(0)) covers them.
    const int n_col = strip * 16 + 4 * j;
    uint32_t sw_bits, st_bits[MT], bias_lo, bias_hi;
    async_load_dword(sw_bits, s_w + n_col / gs);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + r;
        async_load_dword(st_bits[mt], s_tok + (m < M ? m : M - 1));
    }
    // four FP16 bias values; without a bias the loads read a valid dummy address, so that no register
    // with a load in flight ever meets a compiler-made copy at a control-flow merge
    async_load_dword(bias_lo, bias != nullptr ? static_cast<const void *>(bias + n_col) : s_w);
    async_load_dword(bias_hi, bias != nullptr ? static_cast<const void *>(bias + n_col + 2) : s_w);

    auto drain = [&](auto dc) __attribute__((always_inline)) {
        constexpr int d = decltype(dc)::value;
        if constexpr (d < DW) {
            stream_wait<(DW - 1 - d) * LW, LW>(wreg[d]);
            lds_barrier();
            step_compute(wreg[d]);
            ++i;
        }
    };
    static_assert(DW <= 8, "the drain is written out for at most eight stages");
    drain(std::integral_constant<int, 0>{});
    drain(std::integral_constant<int, 1>{});
    drain(std::integral_constant<int, 2>{});
    drain(std::integral_constant<int, 3>{});
    drain(std::integral_constant<int, 4>{});
    drain(std::integral_constant<int, 5>{});
    drain(std::integral_constant<int, 6>{});
    drain(std::integral_constant<int, 7>{});

    // ---- K ranges of one strip: add the accumulators through LDS; range 0 carries on -----------
    // (waves that have ended, the producer among them, no longer count at a barrier)
    if constexpr (Q > 1) {
        lds_barrier();                                // every wave is past its last fragment read: the ring is free
        int32x4 *part = reinterpret_cast<int32x4 *>(smem) + (size_t)cidx * MT * kWave + lane;
        if (q != 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) part[mt * kWave] = acc[mt];
        }
        lds_barrier();
        if (q != 0) return;
#pragma unroll
        for (int o = 1; o < Q; ++o) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] += part[(o * MT + mt) * kWave];
        }
    }

    landed(sw_bits);                                  // the drain ended with vmcnt(0)
    landed(bias_lo);
    landed(bias_hi);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) landed(st_bits[mt]);
    const float sw = __uint_as_float(sw_bits);

    if (WBITS == 4) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[mt][e] >>= 4;   // exact: every product carried the factor 16
    }

    // ---- K split: park the partial strip, count the arrival, last arrival adds the others -----
    if (plan.k_splits > 1) {
        const int nseg = plan.k_splits;
        const size_t slot_ints = (size_t)M * 16;      // one strip of one split
        const __amdgpu_buffer_rsrc_t rs_p = __builtin_amdgcn_make_buffer_rsrc(
            partial, 0, (int)((size_t)plan.strips * nseg * slot_ints * sizeof(int32_t)), kRsrcFlags);
        constexpr int kNowhere = 0x7ffffff0;          // past the end of the buffer: stores dropped, loads 0
        // byte offset of this lane's 16 bytes of row m in the slot of split o
        auto slot_off = [&](int o, int m) __attribute__((always_inline)) {
            return (int)((((size_t)strip * nseg + o) * slot_ints + (size_t)m * 16 + 4 * j) * 4);
        };
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = mt * 16 + r;
            __builtin_amdgcn_raw_buffer_store_b128(acc[mt], rs_p, (m < M) ? slot_off(ks, m) : kNowhere, 0,
                                                   kAuxDeviceCoherent);
        }
        wait_vmcnt<0>();                              // this wave's partial stores are acknowledged
        unsigned prev = 0;
        if (lane == 0)
            prev = __hip_atomic_fetch_add(arrivals + strip, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        prev = __builtin_amdgcn_readfirstlane(prev);
        if (prev != (unsigned)nseg - 1u) return;
        if (lane == 0)                                // leave the counter at zero for the next call
            __hip_atomic_store(arrivals + strip, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int o0 = 0; o0 < nseg; o0 += 4) {        // four partials per round trip
#pragma unroll
            for (int oo = 0; oo < 4; ++oo) {
                const int o = o0 + oo;
                const bool get = o < nseg && o != ks;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int m = mt * 16 + r;
                    acc[mt] += __builtin_amdgcn_raw_buffer_load_b128(rs_p, (get && m < M) ? slot_off(o, m) : kNowhere,
                                                                     0, kAuxDeviceCoherent);
                }
            }
        }
    }

    // ---- dequantize this wave's 16 x (MT*16) strip and write it (App. D epilogue) ---------------
    const half4 bias4 = __builtin_bit_cast(half4, uint2{bias_lo, bias_hi});   // zeros without a bias
    // A lane holds four columns of token r; stored from there, four consecutive lanes would write to
    // four different rows.  One cross-lane permutation per dword puts the 32 contiguous bytes of a
    // token's 16 columns into four consecutive lanes (token lane/4, columns 4*(lane%4)..), which the
    // vector cache handles four times faster.  Every lane computes (rows past M from valid scales,
    // never stored), because the permutation reads all lanes.
    const int pull_out = 4 * ((lane % 4) * 16 + lane / 4);
    const int n_st = strip * 16 + 4 * (lane % 4);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const float sc = __uint_as_float(st_bits[mt]) * sw;
        float f[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[e] = (float)acc[mt][e] * sc;
            if (bias != nullptr) f[e] += (float)bias4[e];
        }
        apply_activation_n<4>(f, act);
        half4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (half_t)f[e];
        uint2 ob = __builtin_bit_cast(uint2, o);
        ob.x = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_out, (int)ob.x);
        ob.y = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_out, (int)ob.y);
        const int m_st = mt * 16 + lane / 4;
        if (m_st < M) *reinterpret_cast<uint2 *>(out + (size_t)m_st * N + n_st) = ob;
        const int m = mt * 16 + r;
        if (acc_out != nullptr && m < M) *reinterpret_cast<int32x4 *>(acc_out + (size_t)m * N + n_col) = acc[mt];
    }
#endif
}

// ---------------------------------------------------------------------------------------------
// The same streaming schedule for FP16 activations x INT8 weights (the W8A16 setting of Sec. 5:
// the input of the QKV GeMM stays FP16).  The weight stream is unchanged (INT8 codes, so half the
// bytes of an FP16 GeMM); each consumer converts the eight bytes of a k step to FP16 in registers
// and multiplies with v_mfma_f32_16x16x32_f16.  The reduction index may be permuted freely as long
// as both operands use the same order, so lane (r, j) feeds bytes 64i + 16j + 8h .. +7 of its
// 16-byte chunk i to k step (i, h) and reads the matching eight FP16 activations, one 16-byte
// LDS read at byte 128i + 32j + 16h of the token's 512-byte stage row.  Accumulation is fp32; with
// a K split the last arrival adds all partials in split order, so the result does not depend on
// arrival order.  Epilogue: acc * s_w[group] + bias (there is no activation scale).
template <int MT, int DW, int R>
__global__ __launch_bounds__(64 * (kMaxConsumers + 1)) void gemm_stream_a16_kernel(
    const half_t *__restrict__ x, const uint8_t *__restrict__ wq, const float *__restrict__ s_w, int gs,
    const half_t *__restrict__ bias, int M, int N, int K, half_t *__restrict__ out, float *__restrict__ partial,
    unsigned *__restrict__ arrivals, StreamPlan plan) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int LW = 4;                             // 16-byte weight loads per lane per stage
    constexpr int X_ROW = kStageK * 2;                // bytes of one token's stage row (FP16)
    constexpr int X_STAGE = MT * 16 * X_ROW;          // bytes of one activation stage
    constexpr int LX = X_STAGE / 1024;                // 1 KB direct loads per stage (producer wave)

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r = lane % 16;
    const int j = lane / 16;

    // blockIdx.x = row block, blockIdx.y = K split; the first `rem` blocks of each kind take one more
    // strip / stage (the quotients come from the host: no integer division at the head of the kernel)
    const int rb = (int)blockIdx.x;
    const int ks = (int)blockIdx.y;
    const int s_lo = rb * plan.strips_per_block + (rb < plan.strips_rem ? rb : plan.strips_rem);
    const int s_hi = s_lo + plan.strips_per_block + (rb < plan.strips_rem ? 1 : 0);
    const int k_lo = ks * plan.stages_per_split + (ks < plan.stages_rem ? ks : plan.stages_rem);
    const int k_hi = k_lo + plan.stages_per_split + (ks < plan.stages_rem ? 1 : 0);
    const int n = k_hi - k_lo;
    const int npad = (n + DW - 1) / DW * DW;

    if (wave == 0) {
        // ---- producer: FP16 activation stages into the LDS ring --------------
        // A 1 KB unit is 2 rows x 512 bytes; 16-byte chunk c of row m sits at position c ^ (m & 15),
        // which makes the consumers' fragment reads (16 rows, one chunk) conflict free.
        const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<half_t *>(x), 0, (int)((size_t)M * K * 2), kRsrcFlags);
        int voff[LX];
#pragma unroll
        for (int u = 0; u < LX; ++u) {
            const int row = u * 2 + lane / 32;
            int grow = row;
            if (grow > M - 1) grow = M - 1;           // rows past M: valid data, results never stored
            voff[u] = grow * K * 2 + (((lane % 32) ^ (row & 15)) * 16);
        }
        auto issue_x = [&](int i, int slot) __attribute__((always_inline)) {
            uint8_t *base = smem + slot * X_STAGE;
            const int soff = (k_lo + i) * X_ROW;
#pragma unroll
            for (int u = 0; u < LX; ++u)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(base + u * 1024), 16, voff[u], soff, 0, 0);
        };
#pragma unroll
        for (int s = 0; s < R - 1; ++s)
            if (s < n) issue_x(s, s);
        for (int i = 0; i < npad; ++i) {
            if (i < n) {
                if (i + R - 2 < n)
                    wait_vmcnt<(R - 2) * LX>();
                else
                    wait_vmcnt<0>();
            }
            lds_barrier();
            if (i + R - 1 < n) issue_x(i + R - 1, (i + R - 1) % R);
        }
        return;
    }

    const int strip = s_lo + wave - 1;
    if (strip >= s_hi) {                              // no strip for this wave: keep the barrier count
        for (int i = 0; i < npad; ++i) lds_barrier();
        return;
    }

    // ---- consumers: INT8 weight strip through registers ----------------------
    const uint32x4 rs_w = make_srd(wq, (uint32_t)((size_t)N * K));
    // Operand layout straight from memory (lane = row r, chunk j).  The chunk-fastest loads of the
    // INT8 kernel measured 5-10 % slower here: the conversion and the twice as large activation
    // fragments already load the vector and LDS pipes that the extra permutations would use.
    const int voff_w = (int)((uint32_t)(strip * 16 + r) * (uint32_t)K + (uint32_t)(j * 16));
    int32x4 wreg[DW][LW];
    auto issue_w = [&](int i, int32x4(&dst)[LW]) __attribute__((always_inline)) {
        if (i > n - 1) i = n - 1;
        const int soff = __builtin_amdgcn_readfirstlane((k_lo + i) * kStageK);
        issue_strip<LW>(dst, voff_w, rs_w, soff);       // same four loads, here in operand order
    };

    float32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = float32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int x_lane = r * X_ROW;
    auto compute = [&](const int32x4(&w)[LW], const uint8_t *xs) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const half8 a = cvt8_i8_f16((uint32_t)w[i][2 * h], (uint32_t)w[i][2 * h + 1]);
                const int c = 8 * i + 2 * j + h;      // 16-byte chunk of the 512-byte row
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const half8 b = *reinterpret_cast<const half8 *>(xs + mt * 16 * X_ROW + x_lane + ((c ^ r) * 16));
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[mt], 0, 0, 0);
                }
            }
        }
    };

    int i = 0;
    auto step_compute = [&](const int32x4(&w)[LW]) __attribute__((always_inline)) {
        if (i < n) compute(w, smem + (i % R) * X_STAGE);
    };
#pragma unroll
    for (int d = 0; d < DW; ++d) issue_w(d, wreg[d]);
    for (int grp = DW; grp < npad; grp += DW) {
#pragma unroll
        for (int d = 0; d < DW; ++d) {
            stream_wait<(DW - 1) * LW, LW>(wreg[d]);
            lds_barrier();
            step_compute(wreg[d]);
            issue_w(i + DW, wreg[d]);
            ++i;
        }
    }
    // epilogue operands fetched under the last stages of the stream (see the INT8 kernel)
    const int n_col = strip * 16 + 4 * j;
    uint32_t sw_bits, bias_lo, bias_hi;
    async_load_dword(sw_bits, s_w + n_col / gs);
    async_load_dword(bias_lo, bias != nullptr ? static_cast<const void *>(bias + n_col) : s_w);
    async_load_dword(bias_hi, bias != nullptr ? static_cast<const void *>(bias + n_col + 2) : s_w);

    auto drain = [&](auto dc) __attribute__((always_inline)) {
        constexpr int d = decltype(dc)::value;
        if constexpr (d < DW) {
            stream_wait<(DW - 1 - d) * LW, LW>(wreg[d]);
            lds_barrier();
            step_compute(wreg[d]);
            ++i;
        }
    };
    static_assert(DW <= 4, "the drain is written out for at most four stages");
    drain(std::integral_constant<int, 0>{});
    drain(std::integral_constant<int, 1>{});
    drain(std::integral_constant<int, 2>{});
    drain(std::integral_constant<int, 3>{});

    landed(sw_bits);                                  // the drain ended with vmcnt(0)
    landed(bias_lo);
    landed(bias_hi);
    const float sw = __uint_as_float(sw_bits);

    // ---- K split: park the fp32 partial strip, count the arrival, last arrival adds all in order --
    if (plan.k_splits > 1) {
        const int nseg = plan.k_splits;
        const size_t slot_words = (size_t)M * 16;
        const __amdgpu_buffer_rsrc_t rs_p = __builtin_amdgcn_make_buffer_rsrc(
            partial, 0, (int)((size_t)plan.strips * nseg * slot_words * sizeof(float)), kRsrcFlags);
        constexpr int kNowhere = 0x7ffffff0;          // past the end of the buffer: stores dropped, loads 0
        auto slot_off = [&](int o, int m) __attribute__((always_inline)) {
            return (int)((((size_t)strip * nseg + o) * slot_words + (size_t)m * 16 + 4 * j) * 4);
        };
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = mt * 16 + r;
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(int32x4, acc[mt]), rs_p,
                                                   (m < M) ? slot_off(ks, m) : kNowhere, 0, kAuxDeviceCoherent);
        }
        wait_vmcnt<0>();
        unsigned prev = 0;
        if (lane == 0)
            prev = __hip_atomic_fetch_add(arrivals + strip, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        prev = __builtin_amdgcn_readfirstlane(prev);
        if (prev != (unsigned)nseg - 1u) return;
        if (lane == 0)
            __hip_atomic_store(arrivals + strip, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = float32x4{0.0f, 0.0f, 0.0f, 0.0f};
        for (int o0 = 0; o0 < nseg; o0 += 4) {        // every partial, this wave's included, in split order
            float32x4 part[4][MT];
#pragma unroll
            for (int oo = 0; oo < 4; ++oo) {
                const int o = o0 + oo;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int m = mt * 16 + r;
                    part[oo][mt] = __builtin_bit_cast(float32x4, __builtin_amdgcn_raw_buffer_load_b128(
                        rs_p, (o < nseg && m < M) ? slot_off(o, m) : kNowhere, 0, kAuxDeviceCoherent));
                }
            }
#pragma unroll
            for (int oo = 0; oo < 4; ++oo)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[mt] += part[oo][mt];
        }
    }

    const half4 bias4 = __builtin_bit_cast(half4, uint2{bias_lo, bias_hi});
    // stores as in the INT8 kernel: a token's 16 columns from four consecutive lanes
    const int pull_out = 4 * ((lane % 4) * 16 + lane / 4);
    const int n_st = strip * 16 + 4 * (lane % 4);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        half4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float f = acc[mt][e] * sw;
            if (bias != nullptr) f += (float)bias4[e];
            o[e] = (half_t)f;
        }
        uint2 ob = __builtin_bit_cast(uint2, o);
        ob.x = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_out, (int)ob.x);
        ob.y = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_out, (int)ob.y);
        const int m_st = mt * 16 + lane / 4;
        if (m_st < M) *reinterpret_cast<uint2 *>(out + (size_t)m_st * N + n_st) = ob;
    }
#endif
}

namespace {

constexpr int kCUs = 256;

int token_tiles(int M) {                          // 16-row token tiles held per consumer: 1, 2, 4 or 8
    const int t = (M + 15) / 16;
    return t > 4 ? 8 : (t > 2 ? 4 : t);
}
int stream_depth(int w_bits) { return w_bits == 8 ? 4 : 8; }   // a stage of a strip is 4 KB (INT8) or 2 KB (INT4)

// Choose the cut (row blocks x K splits) with the lowest modelled time.  The model: a CU streams
// at most kCuRate bytes per microsecond, and no more than its consumers keep in flight over one
// memory latency; the CU with the most bytes sets the time; activation loads share the CU's load
// path in proportion to token tiles per consumer; a K split costs the exchange round trips.
StreamPlan plan_stream(int M, int N, int K, int w_bits, bool allow_split, bool allow_ranges = true) {
    const int S = N / 16, St = K / kStageK, mt = token_tiles(M);
    const double kCuRate = 24e3, kStart = 4.0, kExchange = 4.5, kExchangeRate = 3e6;
    // memory latency in microseconds: about 1 on a quiet chip, 2 with 32 MB streaming, 4 beyond 80 MB
    // (fitted to measured bandwidth against waves per CU)
    double latency = 1.0 + ((double)N * K * w_bits / 8 / 1048576.0 - 8.0) / 24.0;
    latency = latency < 1.0 ? 1.0 : (latency > 4.0 ? 4.0 : latency);
    const double stage_bytes = 16.0 * kStageK * w_bits / 8;      // one strip, one stage
    const double inflight = stream_depth(w_bits) * stage_bytes;   // per consumer wave
    StreamPlan best{S, St, 0, 1, 1};
    double best_t = 1e30;
    // Two K ranges per strip (two waves per strip, accumulators added through LDS): measured to pay
    // for INT8 weights at up to 32 tokens when a CU has at most three strips and the K range of a
    // workgroup is at least 16 stages long (at one token 2048x4096 6.4 -> 5.0 us, 4096x4096 7.6 ->
    // 6.0 us, 12288x4096 13.4 -> 12.1 us); with shorter K or INT4 weights the single producer wave,
    // which then supplies two activation stages per step, and the larger workgroups cost more than
    // the extra streams bring.  They are only weighed against other cuts without a K split, and
    // only given to a cut without one: where the split wins without them it also wins with them
    // (8192-deep 2048x2048: 7.3 us split four ways, 8.3 us with ranges).
    bool ranges_on = false;
    auto range_rule = [&](int c, int st) {
        return (w_bits == 8 && mt <= 2 && st >= 16 && S <= 3 * kCUs && 2 * c <= kMaxConsumers) ? 1 : 0;
    };
    auto range_shift_for = [&](int c, int st) { return ranges_on ? range_rule(c, st) : 0; };
    auto consider = [&](int row_blocks, int k_splits) {
        if (row_blocks < 1 || row_blocks > S || k_splits < 1 || k_splits > St) return;
        const int c = (S + row_blocks - 1) / row_blocks;
        if (c > kMaxConsumers) return;
        if (k_splits > 1 && (!allow_split || S > kMaxSharedStrips)) return;
        if ((double)k_splits * M * N * 4.0 >= 2147483648.0) return;   // 32-bit buffer offsets in the exchange
        const long wgs = (long)row_blocks * k_splits;
        const int per_cu = (int)((wgs + kCUs - 1) / kCUs);
        const int st = (St + k_splits - 1) / k_splits;
        const int waves = c << range_shift_for(c, St / k_splits);   // streams per workgroup
        double rate = waves * per_cu * inflight / latency;
        if (rate > kCuRate) rate = kCuRate;
        const double bytes_cu = (double)per_cu * c * st * stage_bytes * (1.0 + 0.3 * mt / c);
        double t = kStart + bytes_cu / rate;
        if (waves > c) t += 0.3;                    // the accumulators of a strip's ranges meet in LDS
        if (k_splits > 1)                           // round trips, then the partials written and read back
            t += kExchange + 0.3 * k_splits + 2.0 * k_splits * M * N * 4.0 / kExchangeRate;
        // near-ties go to the cut that spreads over more CUs
        const long best_wgs = (long)best.row_blocks * best.k_splits;
        const bool more_cus = (wgs < kCUs ? wgs : kCUs) > (best_wgs < kCUs ? best_wgs : kCUs);
        if (t < best_t * 0.99 || (t < best_t * 1.01 && more_cus)) {
            if (t < best_t) best_t = t;
            best = StreamPlan{S, St, row_blocks, k_splits, c};
        }
    };
    for (int c = 1; c <= kMaxConsumers; ++c) {
        const int row_blocks = (S + c - 1) / c;
        for (int ksp = 1; ksp <= 32; ++ksp) consider(row_blocks, ksp);
    }
    for (int m = 1; m <= 8; ++m)
        for (int ksp = 1; ksp <= 4; ++ksp) consider(kCUs * m / ksp, ksp);   // whole multiples of the CU count
    if (allow_ranges && best.k_splits == 1) {        // second pass: the unsplit cuts again, now with two ranges
        ranges_on = true;
        best_t = 1e30;
        best = StreamPlan{S, St, 0, 1, 1};
        for (int c = 1; c <= kMaxConsumers; ++c) consider((S + c - 1) / c, 1);
        for (int m = 1; m <= 8; ++m) consider(kCUs * m, 1);
    }
    int trb = 0, tks = 0;
    if (tuned_stream_plan(M, N, K, w_bits, &trb, &tks) && (tks == 1 || allow_split))   // validated when registered
        best = StreamPlan{S, St, trb, tks, (S + trb - 1) / trb};
    if (best.row_blocks == 0) {                       // cannot happen (c = 1, no split is always admissible)
        best = StreamPlan{S, St, S, 1, 1};
    }
    best.strips_per_block = S / best.row_blocks;
    best.strips_rem = S % best.row_blocks;
    best.stages_per_split = St / best.k_splits;
    best.stages_rem = St % best.k_splits;
    best.range_shift = (allow_ranges && best.k_splits == 1) ? range_rule(best.consumers, best.stages_per_split) : 0;
    return best;
}

template <int MT, int WBITS, int QSH>
hipError_t launch_stream_q(const GemmArgs &a, const StreamPlan &plan, hipStream_t st) {
    constexpr int R = 3;
    constexpr int DW = (WBITS == 8) ? 4 : 8;
    constexpr size_t lds = ((size_t)R * MT * 16 * kStageK) << QSH;
    static std::atomic<uint64_t> configured{0};
    const void *kernel = reinterpret_cast<const void *>(&gemm_stream_kernel<MT, WBITS, DW, R, QSH>);
    if (hipError_t e = ensure_dynamic_lds(kernel, lds, configured); e != hipSuccess) return e;
    if ((plan.consumers << QSH) > kMaxConsumers) return hipErrorInvalidValue;
    const bool split = plan.k_splits > 1;
    if (split && (a.workspace == nullptr ||
                  a.workspace_bytes < kWsFixedBytes + (size_t)plan.k_splits * a.M * a.N * sizeof(int32_t)))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_stream_kernel<MT, WBITS, DW, R, QSH>), dim3(plan.row_blocks, plan.k_splits),
                       dim3(64 * ((plan.consumers << QSH) + 1)), lds, st, a.xq, a.s_tok,
                       reinterpret_cast<const uint8_t *>(a.wq), a.s_w, a.N / a.groups,
                       reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K, reinterpret_cast<half_t *>(a.out),
                       a.acc_out, split ? reinterpret_cast<int32_t *>(ws_partials(a.workspace)) : nullptr,
                       split ? ws_counters(a.workspace) : nullptr, plan, a.act);
    return hipGetLastError();
}
template <int MT, int WBITS>
hipError_t launch_stream_t(const GemmArgs &a, const StreamPlan &plan, hipStream_t st) {
    if constexpr (WBITS == 8 && MT <= 2) {            // the only combinations the planner gives two ranges
        if (plan.range_shift == 1) return launch_stream_q<MT, WBITS, 1>(a, plan, st);
    }
    if (plan.range_shift != 0) return hipErrorInvalidValue;
    return launch_stream_q<MT, WBITS, 0>(a, plan, st);
}

}  // namespace

// Workspace of the K-split schedule: the fixed part plus one INT32 partial of M x N per split.
// 0 when the chosen cut has no K split.
size_t stream_workspace_bytes(int M, int N, int K, int w_bits) {
    if (K / kStageK < 1) return 0;
    const StreamPlan plan = plan_stream(M, N, K, w_bits, true);
    if (plan.k_splits <= 1) return 0;
    return kWsFixedBytes + (size_t)plan.k_splits * M * N * sizeof(int32_t);
}

void stream_plan(int M, int N, int K, int w_bits, bool allow_split, int *row_blocks, int *k_splits, int *consumers,
                 int *k_ranges) {
    const StreamPlan plan = plan_stream(M, N, K, w_bits, allow_split);
    *row_blocks = plan.row_blocks;
    *k_splits = plan.k_splits;
    *consumers = plan.consumers;
    *k_ranges = 1 << plan.range_shift;
}

namespace {
template <int MT>
hipError_t launch_stream_a16_t(const A16Args &a, const StreamPlan &plan, hipStream_t st) {
    constexpr int R = 3, DW = 4;
    constexpr size_t lds = (size_t)R * MT * 16 * kStageK * 2;
    static std::atomic<uint64_t> configured{0};
    const void *kernel = reinterpret_cast<const void *>(&gemm_stream_a16_kernel<MT, DW, R>);
    if (hipError_t e = ensure_dynamic_lds(kernel, lds, configured); e != hipSuccess) return e;
    const bool split = plan.k_splits > 1;
    if (split && (a.workspace == nullptr ||
                  a.workspace_bytes < kWsFixedBytes + (size_t)plan.k_splits * a.M * a.N * sizeof(float)))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_stream_a16_kernel<MT, DW, R>), dim3(plan.row_blocks, plan.k_splits),
                       dim3(64 * (plan.consumers + 1)), lds, st, reinterpret_cast<const half_t *>(a.x),
                       reinterpret_cast<const uint8_t *>(a.wq), a.s_w, a.N / a.groups,
                       reinterpret_cast<const half_t *>(a.bias), a.M, a.N, a.K, reinterpret_cast<half_t *>(a.out),
                       split ? reinterpret_cast<float *>(ws_partials(a.workspace)) : nullptr,
                       split ? ws_counters(a.workspace) : nullptr, plan);
    return hipGetLastError();
}
}  // namespace

// FP16 activations: the cut of the INT8 call of the same shape (the weight stream is the same), without
// K ranges, which this kernel does not have.  (Weighting the activation tile twice, as its bytes
// would suggest, made the model pick cuts that measured slower; measured better cuts for single
// shapes, e.g. a four-way K split of 4096x4096 at 32 to 64 tokens, can be entered in the schedule table.)
namespace {
StreamPlan plan_stream_a16(int M, int N, int K, bool allow_split) {
    return plan_stream(M, N, K, 8, allow_split, false);
}
}  // namespace

// Workspace of the K-split schedule for FP16 activations: the fixed part plus one fp32 partial of
// M x N per split.
size_t stream_a16_workspace_bytes(int M, int N, int K) {
    if (K / kStageK < 1) return 0;
    const StreamPlan plan = plan_stream_a16(M, N, K, true);
    if (plan.k_splits <= 1) return 0;
    return kWsFixedBytes + (size_t)plan.k_splits * M * N * sizeof(float);
}

void stream_a16_plan(int M, int N, int K, bool allow_split, int *row_blocks, int *k_splits, int *consumers) {
    const StreamPlan plan = plan_stream_a16(M, N, K, allow_split);
    *row_blocks = plan.row_blocks;
    *k_splits = plan.k_splits;
    *consumers = plan.consumers;
}

hipError_t launch_gemm_a16_stream(const A16Args &a, bool allow_split, hipStream_t st) {
    StreamPlan plan = plan_stream_a16(a.M, a.N, a.K, allow_split);
    // never split further than the workspace holds (a schedule-table entry may ask for more splits
    // than the size the caller was told)
    if (plan.k_splits > 1 && kWsFixedBytes + (size_t)plan.k_splits * a.M * a.N * sizeof(float) > a.workspace_bytes)
        plan = plan_stream_a16(a.M, a.N, a.K, false);
    const int mt = token_tiles(a.M);
    if (mt <= 1) return launch_stream_a16_t<1>(a, plan, st);
    if (mt <= 2) return launch_stream_a16_t<2>(a, plan, st);
    return launch_stream_a16_t<4>(a, plan, st);
}

hipError_t launch_gemm_skinny(const GemmArgs &a, bool allow_split, hipStream_t st) {
    const StreamPlan plan = plan_stream(a.M, a.N, a.K, a.w_bits, allow_split);
    const int mt = token_tiles(a.M);
#define ZQ_SK(MT, WB) return launch_stream_t<MT, WB>(a, plan, st)
    if (a.w_bits == 8) {
        if (mt <= 1) ZQ_SK(1, 8);
        if (mt <= 2) ZQ_SK(2, 8);
        if (mt <= 4) ZQ_SK(4, 8);
        ZQ_SK(8, 8);
    } else {
        if (mt <= 1) ZQ_SK(1, 4);
        if (mt <= 2) ZQ_SK(2, 4);
        if (mt <= 4) ZQ_SK(4, 4);
        ZQ_SK(8, 4);
    }
#undef ZQ_SK
}

}  // namespace zq
