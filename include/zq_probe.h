/*
 * zq_probe.h -- measurement probes of libzq (not steps of the quantized layer).
 *
 * The targets for the layer are stated as fractions of two datasheet peaks of the MI355X: INT8
 * matrix-core throughput for large token counts and HBM bandwidth for small ones (Sec. 4.3 names
 * exactly these two regimes: compute-bound large batches, weight-loading-bound small ones).  These
 * calls measure what the installed part sustains for each, so that a benchmark can state every
 * fraction against the datasheet figure and against the measured ceiling.
 *
 * Pointers are DEVICE pointers owned by the caller, 16-byte aligned; nothing is allocated; work is
 * enqueued on `stream`.  Errors: ZQ_ERR_NULL, ZQ_ERR_SHAPE, ZQ_ERR_ALIGN, ZQ_ERR_HIP.
 */
#ifndef ZQ_PROBE_H
#define ZQ_PROBE_H

#include "zq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Read-only stream: every byte of buf[0, bytes) is loaded once (16 bytes per lane, eight workgroups
 * per compute unit, grid stride).  bytes % 16 == 0.  sink: 16 bytes, written only if the data sum
 * to a magic value (never, for practical purposes).  Bandwidth = bytes / kernel time; use a buffer
 * of more than twice the 256 MB last-level cache.
 */
zq_status zq_probe_read_stream(const void *buf, size_t bytes, void *sink, zq_stream stream);

/*
 * Matrix cores alone: `blocks` workgroups of four waves; every wave keeps sixteen 32x32 INT32
 * accumulators and runs iters * 16 v_mfma_i32_32x32x32_i8 on operands that stay in registers.
 *   operands  blocks * 256 * 128 bytes: the eight 16-byte operand fragments of every thread (what the
 *             bytes are decides the figure: the clock follows the power the multipliers draw)
 *   sink      blocks * 256 * 16 bytes
 * Operations = blocks * 4 * iters * 16 * 65536.
 */
zq_status zq_probe_mfma_i8(const void *operands, int blocks, int iters, void *sink, zq_stream stream);

/*
 * Matrix cores fed like the tiled GeMM feeds them: `blocks` workgroups of eight waves (one per compute
 * unit: each takes 128 KB of LDS); every wave runs iters * 32 v_mfma_i32_32x32x32_i8 on the 128 x 64
 * wave tile of the 256 x 256 schedule, reads six 16-byte operand fragments from LDS per eight MFMAs and
 * issues eight 1 KB global -> LDS loads per 32 MFMAs, i.e. the LDS and L2 -> LDS traffic of that
 * schedule's main loop, without its barriers, prologue and epilogue.  The loads cycle through the first
 * 2 MiB of `source` (cache resident), which also supplies the operand bytes; the products mean nothing.
 *   source    at least 2 MiB; what the bytes are decides the figure, as for zq_probe_mfma_i8
 *   sink      blocks * 512 * 16 bytes
 * Operations = blocks * 8 * iters * 32 * 65536.  The result is the rate this tile design can reach on
 * the part when the operand movement shares the chip's power budget with the matrix cores.
 */
zq_status zq_probe_mfma_i8_tile_traffic(const void *source, size_t source_bytes, int blocks, int iters, void *sink,
                                        zq_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* ZQ_PROBE_H */
