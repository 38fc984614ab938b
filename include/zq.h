/*
 * zq.h -- C ABI of libzq: the quantized linear layer of ZeroQuant
 * (arXiv 2206.01861) for AMD MI355X (gfx950).
 *
 * The layer, in the order a transformer block runs it:
 *   1. the FP16 hidden state goes through LayerNorm, or bias-add + GeLU, and
 *      is quantized token by token to INT8 in the same kernel
 *      (Sec. 4.1 "Token-wise Quantization for Activations"; Sec. 4.3 and
 *      App. D "Operation Fusion for Token-wise Activation Quantization");
 *   2. an INT8 x INT8 -> INT32 GeMM runs against weights that were quantized
 *      offline group by group, to INT8 or to INT4 packed two per byte
 *      (Sec. 4.1 "Group-wise Quantization for Weights"; Sec. 4.3 INT8 GeMM);
 *   3. the INT32 accumulator is scaled by the token scale of its row and the
 *      weight-group scale of its column, bias is added, and FP16 is written
 *      once (App. D "Dequantization Associated with GeMM Schedule").
 *
 * Conventions shared by every call
 *   - Every pointer is a DEVICE pointer owned by the caller, valid on the
 *     current HIP device, 16-byte aligned, and sized as documented.  The
 *     library allocates nothing, frees nothing and keeps no device state of
 *     its own: whatever the kernels of one call exchange among themselves
 *     (arrival counters and partial sums of the K-split schedules, the row
 *     maxima of the calls that quantize their output inside the GeMM kernel)
 *     lives in the caller's workspace (see zq_workspace_init).  Calls on
 *     different workspaces are independent and may run at the same time on
 *     different streams.
 *   - Matrices are dense row-major.  "fp16" is IEEE binary16.
 *   - Work is enqueued on `stream` (a hipStream_t; NULL = the default stream)
 *     and the call returns without synchronising.  Outputs must not alias
 *     inputs.  Calls sharing a workspace must be ordered on one stream (or by
 *     events): two of them running at once corrupt each other.
 *   - Arguments are validated on the host before any HIP call; a failed check
 *     returns an error code and launches nothing.  A failed launch returns
 *     ZQ_ERR_HIP.
 *   - Inputs must be finite.  NaN/Inf give unspecified codes, never a fault.
 *
 * The quantizer (App. A.2, uniform symmetric): for a block v sharing a scale,
 *   a = max|v|,  scale = fl32(a / qmax),  inv = fl32(qmax / a),
 *   code = clamp(round_half_even(fl32(v * inv)), -qmax, +qmax),
 *   qmax = 2^(bits-1) - 1  (127 or 7);  a == 0 gives codes 0 and scale 0.
 * The printed S = max(abs(x)) is read as absmax / qmax so that the largest
 * magnitude maps to +-qmax; the code -2^(bits-1) is never produced.
 */
#ifndef ZQ_H
#define ZQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZQ_OK = 0,
    ZQ_ERR_NULL = 1,        /* a required pointer is NULL */
    ZQ_ERR_SHAPE = 2,       /* a dimension is non-positive, not divisible as required, or too large */
    ZQ_ERR_ALIGN = 3,       /* a pointer is not 16-byte aligned */
    ZQ_ERR_UNSUPPORTED = 4, /* bits / dtype / flag value outside the supported set */
    ZQ_ERR_HIP = 5,         /* the HIP runtime reported an error at launch */
    ZQ_ERR_SCRATCH = 6      /* zq_gemm_i8_dequant_static: the shape needs more scratch than the static buffer holds */
} zq_status;

typedef void *zq_stream;

/* Largest reduction length accepted: K * 127 * 127 must stay below 2^31.  With INT4 weights the
 * kernels carry the nibbles as code * 16 and the code -8 is legal input, so K * 127 * 128 must. */
#define ZQ_MAX_K 133143
#define ZQ_MAX_K_W4 132104

/*
 * GeMM workspace.  A workspace is device memory the caller allocates once and hands to the GeMM
 * calls.  Its first ZQ_WORKSPACE_FIXED_BYTES hold what the kernels of a call exchange (control
 * words, 8192 arrival counters, 2^19 eight-byte slots for row maxima); partial sums of the
 * K-split schedules follow.  zq_workspace_init zeroes the fixed part (one small kernel on
 * `stream`, capturable) and must have completed, in stream order, before the first GeMM call
 * that receives the workspace; afterwards only GeMM calls may write to it, and every call leaves
 * the fixed part ready for the next one, whatever its shape or kind.  A workspace that was never
 * initialised, or that something else wrote to, gives undefined results (never a fault).
 * Sizes: zq_gemm_workspace_bytes / zq_gemm_quant_workspace_bytes / zq_gemm_w8a16_workspace_bytes;
 * a buffer of the largest of them over the shapes of a model serves all its calls.
 *   workspace        device, 16-byte aligned;  workspace_bytes >= ZQ_WORKSPACE_FIXED_BYTES
 * Errors: ZQ_ERR_NULL, ZQ_ERR_SHAPE (too small), ZQ_ERR_ALIGN, ZQ_ERR_HIP.
 */
#define ZQ_WORKSPACE_FIXED_BYTES 4227328
zq_status zq_workspace_init(void *workspace, size_t workspace_bytes, zq_stream stream);

const char *zq_status_string(zq_status st);

/* Library version, major*10000 + minor*100 + patch. */
int zq_version(void);

/*
 * Group-wise weight quantization (Sec. 4.1; quantizer of App. A.2).
 *   w_fp16   [N,K] fp16, row = output channel.
 *   groups   g; group j is rows [j*N/g, (j+1)*N/g) over all K columns.
 *            Requires N % g == 0 and (N/g) % 16 == 0 (a group never straddles
 *            a matrix-core tile), K % 16 == 0 (K % 32 == 0 for bits = 4).
 *   bits     8 -> wq_out is int8 [N,K];
 *            4 -> wq_out is uint8 [N,K/2], byte j of row n =
 *                 (code[n,2j] & 0xF) | (code[n,2j+1] << 4), two's complement.
 *   s_w_out  fp32 [g].
 */
zq_status zq_quantize_weight_groupwise(const void *w_fp16, int N, int K, int groups, int bits,
                                       void *wq_out, float *s_w_out, zq_stream stream);

/*
 * LayerNorm fused with token-wise INT8 quantization (Sec. 4.3; App. D).
 *   y[m,:] = (x[m,:] - mean) / sqrt(var + eps) * gamma + beta   (fp32, biased variance)
 *   (xq[m,:], s_tok[m]) = quantizer(y[m,:], qmax 127)
 *   x_fp16 [M,K]; gamma_fp16 [K]; beta_fp16 [K] or NULL; K % 16 == 0, K <= 32768.
 *   xq_out int8 [M,K]; s_tok_out fp32 [M].
 *   y_out  NULL, or [M,K] receiving y before quantization:
 *          y_dtype 0 = fp16 (rounded), 1 = fp32 (exactly the values quantized).
 */
zq_status zq_layernorm_quant_tokenwise(const void *x_fp16, const void *gamma_fp16, const void *beta_fp16,
                                       float eps, int M, int K, int8_t *xq_out, float *s_tok_out,
                                       void *y_out, int y_dtype, zq_stream stream);

/*
 * Bias-add + GeLU fused with token-wise INT8 quantization (Sec. 4.3; App. D).
 *   y = gelu(h + bias);  approx_tanh 0 = erf form, 1 = tanh approximation.
 *   h_fp16 [M,N]; bias_fp16 [N] or NULL; N % 16 == 0, N <= 32768.
 *   Outputs as for the LayerNorm call.
 */
zq_status zq_gelu_quant_tokenwise(const void *h_fp16, const void *bias_fp16, int approx_tanh,
                                  int M, int N, int8_t *xq_out, float *s_tok_out,
                                  void *y_out, int y_dtype, zq_stream stream);

/*
 * Bytes of workspace the GeMM calls can use for (M,N,K) with w_bits in {8,4}.
 * Shapes with few output rows or few output tiles against a long K split the
 * reduction over workgroups and keep INT32 partial sums there (up to 128
 * tokens in the weight-streaming schedule; above that, where 128x128 tiles
 * would occupy less than half the chip, in the tiled schedule, whose epilogue
 * then runs as a second kernel).  The figure is ZQ_WORKSPACE_FIXED_BYTES plus
 * the partial sums, or 0 when no schedule for that shape splits K.  The result
 * of a call never depends on the order in which workgroups finish.
 *
 * zq_gemm_quant_workspace_bytes: the same for a call that also asks for the
 * token-wise quantization of its output (out_q / gq_out): at least
 * ZQ_WORKSPACE_FIXED_BYTES where the GeMM kernel itself would quantize (see
 * zq_gemm_gelu_quant_tokenwise), so never less than zq_gemm_workspace_bytes.
 */
size_t zq_gemm_workspace_bytes(int M, int N, int K, int w_bits);
size_t zq_gemm_quant_workspace_bytes(int M, int N, int K, int w_bits);

/*
 * INT8 GeMM with the dequantization epilogue (Sec. 4.3; App. D).
 *   acc[m,n] = sum_k xq[m,k] * wq[n,k]                          exact, INT32
 *   out[m,n] = fp16( float(acc) * s_tok[m] * s_w[n / (N/groups)] + bias[n] )
 *   xq int8 [M,K]; s_tok fp32 [M]; wq int8 [N,K]; s_w fp32 [groups];
 *   bias_fp16 [N] or NULL; out_fp16 [M,N].
 *   Requires N % groups == 0, (N/groups) % 16 == 0, K % 16 == 0, K <= ZQ_MAX_K (ZQ_MAX_K_W4 with INT4 weights),
 *   and each operand (xq, wq) below 2 GiB (32-bit buffer offsets in the kernels).
 *   acc_out   NULL, or int32 [M,N] receiving the accumulator (parity tap).
 *   out_q / out_s_tok  both NULL, or int8 [M,N] / fp32 [M]: the token-wise
 *             quantization of the FP16-rounded `out`, ready for the next GeMM.
 *   workspace NULL, or an initialised workspace (zq_workspace_init) of
 *             workspace_bytes.  With less than zq_gemm_workspace_bytes(...)
 *             (zq_gemm_quant_workspace_bytes with out_q) the call still
 *             succeeds, on kernels that need none.
 */
zq_status zq_gemm_i8_dequant(const int8_t *xq, const float *s_tok, const int8_t *wq, const float *s_w,
                             int groups, const void *bias_fp16, int M, int N, int K, void *out_fp16,
                             int32_t *acc_out, int8_t *out_q, float *out_s_tok,
                             void *workspace, size_t workspace_bytes, zq_stream stream);

/*
 * zq_gemm_i8_dequant for callers that cannot allocate or be handed device memory beyond their
 * tensors: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments and results as zq_gemm_i8_dequant without the workspace pair: the workspace is a
 * buffer inside the library's code object, ZQ_STATIC_SCRATCH_BYTES (16 MiB) per device, held by every
 * device the library runs on until the process ends.  The call allocates and frees nothing.
 *   - A shape whose schedule would use more workspace than that (zq_gemm_workspace_bytes, or
 *     zq_gemm_quant_workspace_bytes when out_q is given) is refused with ZQ_ERR_SCRATCH and nothing
 *     is launched; zq_gemm_i8_dequant with a caller's workspace takes such shapes.
 *   - All calls of this entry point on one device share that device's buffer, and the buffer keeps
 *     what the last call left (the kernels leave the control words, counters and slots ready for the
 *     next call; partial sums are overwritten before they are read).  Calls must therefore be
 *     ordered, on one stream or by events: two of them running at once on one device race.
 * Other errors as zq_gemm_i8_dequant.
 */
#define ZQ_STATIC_SCRATCH_BYTES 16777216
zq_status zq_gemm_i8_dequant_static(const int8_t *xq, const float *s_tok, const int8_t *wq, const float *s_w,
                                    int groups, const void *bias_fp16, int M, int N, int K, void *out_fp16,
                                    int32_t *acc_out, int8_t *out_q, float *out_s_tok, zq_stream stream);

/*
 * Same layer with INT4 weights (the W4/8 policy of Sec. 5 puts INT4 on the
 * feed-forward weights).  wq4 is uint8 [N,K/2] in the packing documented at
 * zq_quantize_weight_groupwise; K % 32 == 0.  acc_out holds the product of
 * the INT8 activation codes with the sign-extended INT4 codes.
 */
zq_status zq_gemm_w4a8_dequant(const int8_t *xq, const float *s_tok, const uint8_t *wq4, const float *s_w,
                               int groups, const void *bias_fp16, int M, int N, int K, void *out_fp16,
                               int32_t *acc_out, int8_t *out_q, float *out_s_tok,
                               void *workspace, size_t workspace_bytes, zq_stream stream);

/*
 * The two operators of the unfused pipeline (Fig. 2, left; App. D describes
 * the stand-alone quantization operator that the fused kernels replace), kept
 * as calls of their own: for layers whose producer is not LayerNorm or GeLU,
 * and to measure what the fusions save.
 *
 * zq_quantize_tokenwise: token-wise INT8 quantization (App. A.2, one scale per
 * row) of an FP16 tensor.
 *   x_fp16   in,  fp16 [M,K] row-major (device)
 *   xq_out   out, int8 [M,K];  s_tok_out  out, fp32 [M]  (device)
 * K % 16 == 0, K <= 32768.  Errors as zq_layernorm_quant_tokenwise.
 *
 * zq_dequantize_acc: out[m,n] = fp16( acc[m,n] * s_tok[m] * s_w[n / (N/groups)] + bias[n] ),
 * the dequantization epilogue of App. D as a kernel of its own (fp32
 * arithmetic, one FP16 rounding; agrees with the GeMM calls' output for the
 * same acc to within one FP16 step).
 *   acc      in,  int32 [M,N] (device);  s_tok fp32 [M];  s_w fp32 [groups];  bias_fp16 fp16 [N] or NULL
 *   out_fp16 out, fp16 [M,N] (device)
 * N % groups == 0, (N/groups) % 16 == 0.  ZQ_ERR_NULL / ZQ_ERR_SHAPE / ZQ_ERR_ALIGN as elsewhere.
 */
zq_status zq_quantize_tokenwise(const void *x_fp16, int M, int K, int8_t *xq_out, float *s_tok_out, zq_stream stream);
zq_status zq_dequantize_acc(const int32_t *acc, const float *s_tok, const float *s_w, int groups,
                            const void *bias_fp16, int M, int N, void *out_fp16, zq_stream stream);

/*
 * First feed-forward GeMM with the activation in its epilogue (Sec. 4.3 and
 * App. D fuse bias-add + GeLU with the token-wise quantization that feeds the
 * second GeMM; here the bias-add and the GeLU move one step earlier, into the
 * dequantization epilogue of the first GeMM, so the activation tensor is
 * written once, already activated):
 *   g[m,n]    = fp16( GeLU( acc[m,n] * s_tok[m] * s_w[n / (N/groups)] + bias[n] ) )
 *   (gq, s')  = token-wise INT8 quantization (App. A.2, per row of g) of g as stored in FP16
 * GeLU is evaluated in fp32 on the unrounded dequantized value (erf form, or
 * the tanh form when approx_tanh = 1), which differs from the two-call chain
 * zq_gemm_*_dequant -> zq_gelu_quant_tokenwise only by that one FP16 rounding
 * of the pre-activation.  The INT32 accumulator is not exported.
 *   xq, s_tok, s_w, groups, bias_fp16, M, N, K, workspace: as zq_gemm_i8_dequant
 *   wq        w_bits = 8: int8 [N,K];  w_bits = 4: packed uint8 [N,K/2]   (device)
 *   g_fp16    out, fp16 [M,N]: the activated tensor (device); may be NULL
 *             when zq_gemm_quantizes_in_kernel() says 1 for the shape (the
 *             tensor is then never written), otherwise ZQ_ERR_UNSUPPORTED
 *   gq_out    out, int8 [M,N];  s_tok_out  out, fp32 [M]                  (device, required)
 * N <= 32768 (a row of g is quantized from registers).  Errors as the GeMM calls.
 *
 * Where the quantization happens.  On the tiled schedules (large token counts)
 * the GeMM kernel itself quantizes when the call has a workspace: the tiles
 * that share a band of token rows exchange their row maxima through the
 * workspace, wait for each other, and write the codes from their accumulator
 * registers, so g is not read back (and not written at all when g_fp16 is
 * NULL).  The same holds for out_q / out_s_tok of zq_gemm_i8_dequant and
 * zq_gemm_w4a8_dequant.  Elsewhere, and without a workspace, a second kernel
 * quantizes the FP16 rows just written.  Both ways give the same bits.  It
 * needs a band of tiles to fit a quarter of the device's compute units (N <=
 * 16384 on 256 of them) and (M rounded up to the tile edge) * (tiles along N)
 * <= 2^19 exchange slots; beyond that the second kernel is used.
 * The wait of a tile for its band is bounded (about a second).  It cannot run
 * out while workgroups are started in id order, which is how the hardware
 * dispatches them; if it does all the same, the rows concerned come back with
 * out_s_tok = NaN and codes -128 (a value the quantizer never produces) in the
 * columns of the tiles that gave up, and zq_quant_wait_expired counts it.
 */
zq_status zq_gemm_gelu_quant_tokenwise(const int8_t *xq, const float *s_tok, const void *wq, int w_bits,
                                       const float *s_w, int groups, const void *bias_fp16, int approx_tanh, int M,
                                       int N, int K, void *g_fp16, int8_t *gq_out, float *s_tok_out,
                                       void *workspace, size_t workspace_bytes, zq_stream stream);

/*
 * W8A16 GeMM (Sec. 5: for the largest model the input of the QKV GeMM stays
 * FP16 while the weights are INT8): FP16 activations against group-wise INT8
 * weights (App. A.2), fp32 accumulation, weight-scale epilogue
 *   out[m,n] = fp16( (sum_k x[m,k] * wq[n,k]) * s_w[n / (N/groups)] + bias[n] ).
 *   x_fp16    in,  fp16 [M,K] row-major                      (device)
 *   wq        in,  int8 [N,K];  s_w  fp32 [groups];  bias_fp16  fp16 [N] or NULL   (device)
 *   out_fp16  out, fp16 [M,N]                                (device)
 *   workspace an initialised workspace (zq_workspace_init) of zq_gemm_w8a16_workspace_bytes(M, N, K)
 *             bytes, or NULL: lets small token counts split K across workgroups where that is
 *             faster (fp32 partials; the result does not depend on the order in which workgroups finish)
 * K % 16 == 0, K <= ZQ_MAX_K, N % groups == 0, (N/groups) % 16 == 0 (up to 128 tokens the streaming
 * schedule needs K % 256 == 0, and 65 to 128 tokens run as two launches of it over row halves unless
 * the tiled schedule with a K split is the faster choice for the shape and the workspace allows it;
 * other small shapes run an untiled schedule).  The codes are converted to
 * FP16 exactly; the sum is accumulated in fp32 on the FP16 matrix cores, so unlike the INT8 calls
 * the result is reproducible but not bit-defined by the inputs alone (tolerance in the tests).
 * Errors: ZQ_ERR_NULL, ZQ_ERR_SHAPE, ZQ_ERR_ALIGN, ZQ_ERR_HIP.
 */
zq_status zq_gemm_w8a16_dequant(const void *x_fp16, const int8_t *wq, const float *s_w, int groups,
                                const void *bias_fp16, int M, int N, int K, void *out_fp16, void *workspace,
                                size_t workspace_bytes, zq_stream stream);

/*
 * Workspace that lets zq_gemm_w8a16_dequant split K for this shape (0: the call never splits),
 * and the cut its streaming schedule takes for up to 64 tokens (arguments and
 * results as zq_gemm_stream_plan; the cut is the INT8 call's unless that one divides strips into
 * K ranges, which this schedule does not do).  Host-only; launch nothing.
 */
size_t zq_gemm_w8a16_workspace_bytes(int M, int N, int K);
int zq_gemm_w8a16_stream_plan(int M, int N, int K, size_t workspace_bytes, int *row_blocks, int *k_splits,
                              int *consumers);

/*
 * Tuning and test hook: force the GeMM schedule instead of choosing it from
 * the shape (App. D picks a schedule by batch x sequence length).
 * variant < 0 restores automatic choice.  A forced schedule whose shape
 * constraints are not met returns ZQ_ERR_UNSUPPORTED from the GeMM call.
 * Process-wide; not for concurrent use.  Returns the previous value.
 */
int zq_debug_force_gemm_variant(int variant);

/*
 * 1 if a GeMM call with out_q / gq_out on this shape quantizes its output
 * inside the GeMM kernel (see zq_gemm_gelu_quant_tokenwise), else 0.
 *
 * zq_debug_set_in_kernel_quant: test and ablation hook; on = 0 makes every
 * call use the second kernel.  Process-wide; returns the previous value.
 *
 * zq_quant_wait_expired: *count_out receives the number of threads (one per
 * tile and token row) whose bounded wait ran out in calls on this workspace
 * since the last call of this function, 0 in every correct run, and the
 * count is reset.  Synchronous: it copies one word from the device, so every
 * call on the workspace must have been waited for.  ZQ_ERR_NULL, ZQ_ERR_ALIGN,
 * ZQ_ERR_HIP.
 */
int zq_gemm_quantizes_in_kernel(int M, int N, int K, int w_bits, size_t workspace_bytes);
int zq_debug_set_in_kernel_quant(int on);
zq_status zq_quant_wait_expired(void *workspace, int *count_out);

/* Name of schedule `variant` (NULL when out of range), and the schedule the
 * dispatcher would choose for a shape. */
const char *zq_gemm_variant_name(int variant);
int zq_gemm_choose_variant(int M, int N, int K, int w_bits, size_t workspace_bytes);

/*
 * Measured schedule table (App. D ranks schedules by measuring them offline
 * and picks by batch x sequence length at run time).  zq_tune_set registers,
 * for the GeMM shape (N, K, w_bits) and token counts m_lo..m_hi, the schedule
 * `variant` to use instead of the built-in choice and, for the two streaming
 * schedules, the cut (row_blocks, k_splits; both 0 = keep the cost model's).
 * An entry is ignored for a call whose workspace cannot hold its K split.
 * The latest matching entry wins.  zq_gemm_workspace_bytes, zq_gemm_choose_variant
 * and zq_gemm_stream_plan reflect the table.  Process-wide; not for use
 * concurrently with GeMM calls.  The Python module paper_2206_01861_amd.autotune
 * fills the table by timing the candidates on the installed GPU.
 * Returns ZQ_OK, ZQ_ERR_SHAPE (ranges, or a cut the kernels cannot run:
 * more than eight strips per row block, more splits than stages, ...),
 * ZQ_ERR_UNSUPPORTED (unknown variant, a cut for a non-streaming schedule).
 */
int zq_tune_set(int m_lo, int m_hi, int N, int K, int w_bits, int variant, int row_blocks, int k_splits);
void zq_tune_clear(void);
int zq_tune_count(void);

/*
 * How the weight-streaming schedules (M <= 128, K a multiple of 256) cut a
 * GeMM over the chip (Sec. 4.3: small-batch latency is weight-loading time,
 * so the cut is made for memory bandwidth): the N/16 strips of 16 weight rows
 * are dealt evenly over *row_blocks workgroups of *consumers strips at most,
 * and K is divided over *k_splits workgroups (1 unless a workspace of at
 * least zq_gemm_workspace_bytes() is offered and the matrix has too few rows
 * to occupy every CU otherwise).  Host-only; launches nothing.
 * Returns ZQ_OK, ZQ_ERR_NULL, or ZQ_ERR_UNSUPPORTED for a shape these
 * schedules do not take.
 */
int zq_gemm_stream_plan(int M, int N, int K, int w_bits, size_t workspace_bytes, int *row_blocks, int *k_splits,
                        int *consumers);

/*
 * Into how many K ranges the streaming schedule divides each strip inside a
 * workgroup for the cut zq_gemm_stream_plan reports: 1, or 2 (INT8 weights, at
 * most 32 tokens, no K split, few strips per CU and K of 4096 or more: each
 * strip is then streamed by two waves over halves of K, which doubles the
 * loads a CU keeps in flight, and their INT32 accumulators are added before
 * the epilogue, so results do not change).  Host-only; launches nothing.
 * Returns 0 for a shape these schedules do not take.
 */
int zq_gemm_stream_k_ranges(int M, int N, int K, int w_bits, size_t workspace_bytes);

#ifdef __cplusplus
}
#endif
#endif /* ZQ_H */
