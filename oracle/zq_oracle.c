/*
 * zq_oracle.c -- plain CPU oracle for the ZeroQuant quantized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or constant with the HIP path and must never be called from
 * the product path; only tests, the smoke check and the cpu_baseline leg of
 * the benchmark may load it.
 *
 * What it follows (ZeroQuant, arXiv 2206.01861):
 *   - uniform symmetric scalar quantizer         App. A.2 (unnumbered equation)
 *   - group-wise weight quantization             Sec. 4.1, "Group-wise Quantization for Weights"
 *   - token-wise dynamic activation quantization Sec. 4.1, "Token-wise Quantization for Activations"
 *   - LayerNorm / bias+GeLU feeding the quantizer Sec. 4.3 and App. D, "Operation Fusion ..."
 *   - INT8 x INT8 -> INT32 GeMM                  Sec. 4.3 "CUTLASS INT8 GeMM", App. D
 *   - dequantization of the INT32 accumulator with the token (row) and the
 *     weight-group (column) scale                App. D, "Dequantization Associated with GeMM Schedule"
 *
 * Readings where the paper is silent or under-specified (each is repeated at
 * the function that uses it):
 *   R1  scale  S = absmax / (2^(bit-1) - 1), so that absmax maps to +-qmax.
 *       App. A.2 prints S = max(abs(x)); taken literally all codes would be
 *       -1/0/1, so the missing level count is restored.
 *   R2  codes are clamped to [-qmax, +qmax] (the value -2^(bit-1) of the
 *       printed clamp range cannot be reached under R1).
 *   R3  "round" is round-half-to-even.
 *   R4  x/S is evaluated as x * inv with inv = fl32(qmax / absmax); the stored
 *       scale is fl32(absmax / qmax).  One IEEE fp32 divide each, one fp32
 *       multiply per element, no fused multiply-add.
 *   R5  a group is N/g consecutive output rows over all K columns.
 *   R6  all-zero row/group: codes 0, scale 0.
 *   R7  LayerNorm: biased variance, eps inside the square root, affine
 *       gamma (required) and beta (optional); evaluated in fp64.
 *   R8  GeLU: erf form, or the tanh approximation on request; fp64.
 *   R9  INT4: two's-complement nibbles, even k in the low nibble.
 *
 * Floating point is fp64 wherever the paper does not fix a precision; the
 * quantizer itself is fp32 by reading R4 because there floating point decides
 * an integer and both sides must take that decision in the same precision.
 *
 * Parity pins live in tests/test_oracle_*.py (invariants, closed forms,
 * brute force, library special cases).  The paper prints no worked numeric
 * example for any of these functions.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- fp16 bit pattern -> float, exact ---------------------------------- */
static float half_bits_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t expo = (uint32_t)(h >> 10) & 0x1fu;
    uint32_t mant = (uint32_t)h & 0x3ffu;
    float v;
    if (expo == 0) {
        v = ldexpf((float)mant, -24);              /* zero or subnormal */
    } else if (expo == 31) {
        v = mant ? NAN : INFINITY;
    } else {
        v = ldexpf((float)(mant | 0x400u), (int)expo - 25);
    }
    return sign ? -v : v;
}

void zq_oracle_half_to_float(const uint16_t *h, long n, float *out)
{
    for (long i = 0; i < n; ++i) out[i] = half_bits_to_float(h[i]);
}

/* ---- the quantizer (App. A.2 with readings R1-R4, R6) ------------------- */
/* v: n fp32 values sharing one scale.  q: n codes.  returns the scale. */
static float quantize_block(const float *v, long n, int qmax, int8_t *q)
{
    float a = 0.0f;
    for (long i = 0; i < n; ++i) {
        float t = fabsf(v[i]);
        if (t > a) a = t;
    }
    if (a == 0.0f) {
        for (long i = 0; i < n; ++i) q[i] = 0;
        return 0.0f;
    }
    volatile float scale = a / (float)qmax;   /* volatile: force fp32 rounding */
    volatile float inv = (float)qmax / a;
    for (long i = 0; i < n; ++i) {
        volatile float t = v[i] * inv;
        float r = nearbyintf(t);              /* default mode: ties to even */
        if (r > (float)qmax) r = (float)qmax;
        if (r < -(float)qmax) r = -(float)qmax;
        q[i] = (int8_t)r;
    }
    return scale;
}

/* One scale per row: y32 [M,K] -> xq int8 [M,K], s_tok [M].
 * Sec. 4.1 token-wise quantization, 8 bit. */
void zq_oracle_quant_tokenwise(const float *y32, long M, long K,
                               int8_t *xq, float *s_tok)
{
    #pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m)
        s_tok[m] = quantize_block(y32 + m * K, K, 127, xq + m * K);
}

/* Generic entry used by the pins: one block, any qmax. */
float zq_oracle_quantize_block(const float *v, long n, int qmax, int8_t *q)
{
    return quantize_block(v, n, qmax, q);
}

/* ---- group-wise weight quantization (Sec. 4.1; R5, R9) ------------------ */
/* w: fp16 bit patterns [N,K] row-major, row = output channel.
 * bits = 8: wq is int8 [N,K].  bits = 4: wq is uint8 [N,K/2] packed.
 * codes_out (nullable): unpacked int8 codes [N,K] in either case.
 * returns 0, or -1 on a bad argument. */
int zq_oracle_quantize_weight_groupwise(const uint16_t *w, long N, long K,
                                        long groups, int bits,
                                        void *wq, float *s_w, int8_t *codes_out)
{
    if (N <= 0 || K <= 0 || groups <= 0 || N % groups) return -1;
    if (bits != 8 && bits != 4) return -1;
    if (bits == 4 && (K & 1)) return -1;
    const int qmax = (bits == 8) ? 127 : 7;
    const long gs = N / groups;
    const long blk = gs * K;
    #pragma omp parallel for schedule(static)
    for (long j = 0; j < groups; ++j) {
        float *v = (float *)malloc(sizeof(float) * (size_t)blk);
        int8_t *q = (int8_t *)malloc((size_t)blk);
        for (long i = 0; i < blk; ++i) v[i] = half_bits_to_float(w[j * blk + i]);
        s_w[j] = quantize_block(v, blk, qmax, q);
        if (codes_out) memcpy(codes_out + j * blk, q, (size_t)blk);
        if (bits == 8) {
            memcpy((int8_t *)wq + j * blk, q, (size_t)blk);
        } else {
            uint8_t *p = (uint8_t *)wq + j * blk / 2;
            for (long i = 0; i < blk / 2; ++i)
                p[i] = (uint8_t)(((uint8_t)q[2 * i] & 0x0fu) |
                                 (((uint8_t)q[2 * i + 1] & 0x0fu) << 4));
        }
        free(v);
        free(q);
    }
    return 0;
}

/* packed uint8 [n_bytes] -> int8 codes [2*n_bytes]  (R9) */
void zq_oracle_unpack_int4(const uint8_t *packed, long n_bytes, int8_t *codes)
{
    for (long i = 0; i < n_bytes; ++i) {
        int lo = packed[i] & 0x0f;
        int hi = (packed[i] >> 4) & 0x0f;
        codes[2 * i] = (int8_t)(lo >= 8 ? lo - 16 : lo);
        codes[2 * i + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
    }
}

/* ---- LayerNorm in fp64 (R7) --------------------------------------------- */
/* x fp16 [M,K]; gamma fp16 [K]; beta fp16 [K] or NULL.
 * y64 (nullable) [M,K] fp64; y32 (nullable) [M,K] = (float)y64. */
void zq_oracle_layernorm(const uint16_t *x, const uint16_t *gamma,
                         const uint16_t *beta, double eps, long M, long K,
                         double *y64, float *y32)
{
    #pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        const uint16_t *row = x + m * K;
        double sum = 0.0;
        for (long k = 0; k < K; ++k) sum += (double)half_bits_to_float(row[k]);
        const double mean = sum / (double)K;
        double ss = 0.0;
        for (long k = 0; k < K; ++k) {
            double d = (double)half_bits_to_float(row[k]) - mean;
            ss += d * d;
        }
        const double var = ss / (double)K;
        const double rstd = 1.0 / sqrt(var + eps);
        for (long k = 0; k < K; ++k) {
            double d = (double)half_bits_to_float(row[k]) - mean;
            double y = d * rstd * (double)half_bits_to_float(gamma[k]);
            if (beta) y += (double)half_bits_to_float(beta[k]);
            if (y64) y64[m * K + k] = y;
            if (y32) y32[m * K + k] = (float)y;
        }
    }
}

/* ---- bias + GeLU in fp64 (R8) ------------------------------------------- */
/* h fp16 [M,N]; bias fp16 [N] or NULL; approx_tanh selects the tanh form. */
void zq_oracle_gelu(const uint16_t *h, const uint16_t *bias, int approx_tanh,
                    long M, long N, double *y64, float *y32)
{
    const double inv_sqrt2 = 0.70710678118654752440;
    const double sqrt_2_over_pi = 0.79788456080286535588;
    #pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        for (long n = 0; n < N; ++n) {
            double u = (double)half_bits_to_float(h[m * N + n]);
            if (bias) u += (double)half_bits_to_float(bias[n]);
            double y;
            if (approx_tanh)
                y = 0.5 * u * (1.0 + tanh(sqrt_2_over_pi * (u + 0.044715 * u * u * u)));
            else
                y = 0.5 * u * (1.0 + erf(u * inv_sqrt2));
            if (y64) y64[m * N + n] = y;
            if (y32) y32[m * N + n] = (float)y;
        }
    }
}

/* ---- GeLU of fp64 values (the activation of Sec. 4.3's fused bias-add + GeLU,
 * applied to an already dequantized pre-activation) ------------------------- */
/* u fp64 [n] -> y fp64 [n]; approx_tanh selects the tanh form. */
void zq_oracle_gelu_f64(const double *u, int approx_tanh, long n, double *y)
{
    const double inv_sqrt2 = 0.70710678118654752440;
    const double sqrt_2_over_pi = 0.79788456080286535588;
    #pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) {
        const double v = u[i];
        if (approx_tanh)
            y[i] = 0.5 * v * (1.0 + tanh(sqrt_2_over_pi * (v + 0.044715 * v * v * v)));
        else
            y[i] = 0.5 * v * (1.0 + erf(v * inv_sqrt2));
    }
}

/* ---- exact integer GeMM (Sec. 4.3 / App. D) ------------------------------ */
/* acc[m,n] = sum_k xq[m,k] * wq[n,k], int32 accumulation. */
void zq_oracle_matmul_i32(const int8_t *xq, const int8_t *wq,
                          long M, long N, long K, int32_t *acc)
{
    #pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        for (long n = 0; n < N; ++n) {
            int32_t s = 0;
            for (long k = 0; k < K; ++k)
                s += (int32_t)xq[m * K + k] * (int32_t)wq[n * K + k];
            acc[m * N + n] = s;
        }
    }
}

/* Same sum carried in int64: shows the int32 result did not wrap. */
void zq_oracle_matmul_i64(const int8_t *xq, const int8_t *wq,
                          long M, long N, long K, int64_t *acc)
{
    #pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        for (long n = 0; n < N; ++n) {
            int64_t s = 0;
            for (long k = 0; k < K; ++k)
                s += (int64_t)xq[m * K + k] * (int64_t)wq[n * K + k];
            acc[m * N + n] = s;
        }
    }
}

/* Selected rows only: rows[i] indexes xq; acc is [n_rows,N]. */
void zq_oracle_matmul_i32_rows(const int8_t *xq, const int8_t *wq,
                               const long *rows, long n_rows,
                               long N, long K, int32_t *acc)
{
    #pragma omp parallel for schedule(static) collapse(2)
    for (long i = 0; i < n_rows; ++i) {
        for (long n = 0; n < N; ++n) {
            const int8_t *xr = xq + rows[i] * K;
            int32_t s = 0;
            for (long k = 0; k < K; ++k)
                s += (int32_t)xr[k] * (int32_t)wq[n * K + k];
            acc[i * N + n] = s;
        }
    }
}

/* ---- FP16 activations x INT8 weights (the W8A16 setting of Sec. 5: the input of the
 * QKV GeMM stays FP16, the weights are INT8 codes with group-wise scales) ---- */
/* acc[m,n] = sum_k x[m,k] * wq[n,k] in fp64 (every product is exact in fp64);
 * absacc (nullable) = sum_k |x[m,k]| * |wq[n,k]|, the size of the terms that were added.
 * rows (nullable): only these rows of x, acc is then [n_rows,N]. */
void zq_oracle_matmul_f16_i8(const uint16_t *x, const int8_t *wq, const long *rows, long n_rows,
                             long N, long K, double *acc, double *absacc)
{
    #pragma omp parallel for schedule(static) collapse(2)
    for (long i = 0; i < n_rows; ++i) {
        for (long n = 0; n < N; ++n) {
            const uint16_t *xr = x + (rows ? rows[i] : i) * K;
            double s = 0.0, a = 0.0;
            for (long k = 0; k < K; ++k) {
                const double p = (double)half_bits_to_float(xr[k]) * (double)wq[n * K + k];
                s += p;
                a += fabs(p);
            }
            acc[i * N + n] = s;
            if (absacc) absacc[i * N + n] = a;
        }
    }
}

/* ref[m,n] = acc[m,n] * s_w[n / (N/groups)] + bias[n]; mag (nullable) = |acc*s_w| + |bias|. */
void zq_oracle_dequant_w(const double *acc, const float *s_w, long groups, const uint16_t *bias,
                         long M, long N, double *ref, double *mag)
{
    const long gs = N / groups;
    #pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        for (long n = 0; n < N; ++n) {
            const double t = acc[m * N + n] * (double)s_w[n / gs];
            const double b = bias ? (double)half_bits_to_float(bias[n]) : 0.0;
            ref[m * N + n] = t + b;
            if (mag) mag[m * N + n] = fabs(t) + fabs(b);
        }
    }
}

/* ---- dequantization (App. D) --------------------------------------------- */
/* ref[m,n] = acc * s_tok[m] * s_w[n / (N/groups)] + bias[n], in fp64.
 * mag (nullable) = |acc*s_tok*s_w| + |bias|, the magnitude the relative
 * tolerance of the fp16 output is taken against. */
void zq_oracle_dequant(const int32_t *acc, const float *s_tok, const float *s_w,
                       long groups, const uint16_t *bias, long M, long N,
                       double *ref, double *mag)
{
    const long gs = N / groups;
    #pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        for (long n = 0; n < N; ++n) {
            double p = (double)acc[m * N + n] * (double)s_tok[m] * (double)s_w[n / gs];
            double b = bias ? (double)half_bits_to_float(bias[n]) : 0.0;
            ref[m * N + n] = p + b;
            if (mag) mag[m * N + n] = fabs(p) + fabs(b);
        }
    }
}
