"""Pins for the oracle's integer GeMM and dequantization (Sec. 4.3, App. D).

The GeMM reaches exactly the integer matrix product, so the oracle is that
definition; it is pinned against closed forms, a pure-Python triple loop on
tiny inputs, numpy's int64 matmul, and structure tests that a transposed
operand or a wrong stride would fail.
"""
import numpy as np
import pytest

import zq_inputs
from oracle import zq_oracle as orc


def test_tiny_products_against_python_triple_loop():
    rng = zq_inputs.rng_for(8, 1)
    for (M, N, K) in [(1, 1, 1), (2, 3, 5), (3, 2, 64), (8, 8, 48), (5, 7, 17)]:
        x = zq_inputs.random_codes(rng, (M, K))
        w = zq_inputs.random_codes(rng, (N, K))
        acc = orc.matmul_i32(x, w)
        xl, wl = x.tolist(), w.tolist()
        for m in range(M):
            for n in range(N):
                assert acc[m, n] == sum(xl[m][k] * wl[n][k] for k in range(K))


@pytest.mark.parametrize("M,N,K", [(7, 48, 256), (33, 80, 768), (129, 16, 1024)])
def test_against_numpy_int64_matmul_and_no_wrap(M, N, K):
    rng = zq_inputs.rng_for(8, 2)
    x = zq_inputs.random_codes(rng, (M, K))
    w = zq_inputs.random_codes(rng, (N, K))
    want = x.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(orc.matmul_i32(x, w).astype(np.int64), want)
    assert np.array_equal(orc.matmul_i64(x, w), want)
    rows = np.array([0, M - 1, M // 2])
    assert np.array_equal(orc.matmul_i32_rows(x, w, rows).astype(np.int64), want[rows])


def test_closed_forms():
    # all codes 127: acc = 127^2 * K, at the largest K of the workloads
    K = 24576
    x = np.full((2, K), 127, np.int8)
    w = np.full((3, K), 127, np.int8)
    assert (orc.matmul_i32(x, w) == 16129 * K).all()
    assert 16129 * K == 396386304 < 2 ** 31
    w[1] = -127
    assert (orc.matmul_i32(x, w)[:, 1] == -16129 * K).all()
    # a selector weight (one 1 per row) copies columns of x: catches transposes/strides
    rng = zq_inputs.rng_for(8, 3)
    x = zq_inputs.random_codes(rng, (5, 32))
    sel = np.zeros((32, 32), np.int8)
    perm = rng.permutation(32)
    sel[np.arange(32), perm] = 1
    assert np.array_equal(orc.matmul_i32(x, sel), x[:, perm].astype(np.int32))
    # rank-one: acc[m,n] = K * a[m] * b[n]
    a = np.array([1, -2, 3], np.int8)
    b = np.array([4, 5, -6, 7], np.int8)
    x = np.repeat(a[:, None], 16, axis=1)
    w = np.repeat(b[:, None], 16, axis=1)
    assert np.array_equal(orc.matmul_i32(x, w), 16 * np.outer(a.astype(np.int32), b.astype(np.int32)))


def test_int4_weights_product_goes_through_unpacked_codes():
    rng = zq_inputs.rng_for(8, 4)
    w16 = zq_inputs.weights(rng, 32, 64)
    wq4, s_w, codes = orc.quantize_weight_groupwise(w16, 2, 4)
    x = zq_inputs.random_codes(rng, (6, 64))
    acc = orc.matmul_i32(x, orc.unpack_int4(wq4))
    assert np.array_equal(acc.astype(np.int64), x.astype(np.int64) @ codes.astype(np.int64).T)


def test_dequant_hand_example_and_broadcast():
    acc = np.array([[100, -200, 300, 400], [1, 2, 3, 4]], np.int32)
    s_tok = np.array([0.5, 2.0], np.float32)
    s_w = np.array([0.25, 0.125], np.float32)        # groups of 2 columns
    bias = np.array([1.0, -1.0, 0.5, 0.0], np.float16)
    ref, mag = orc.dequant(acc, s_tok, s_w, bias)
    want = np.array([[100 * .5 * .25 + 1, -200 * .5 * .25 - 1, 300 * .5 * .125 + .5, 400 * .5 * .125],
                     [1 * 2 * .25 + 1, 2 * 2 * .25 - 1, 3 * 2 * .125 + .5, 4 * 2 * .125]])
    assert np.array_equal(ref, want)
    assert mag[0, 1] == 25.0 + 1.0
    ref2, _ = orc.dequant(acc, s_tok, s_w, None)
    assert np.array_equal(ref2, want - bias.astype(np.float64)[None, :])
    # random: equals numpy broadcasting in fp64
    rng = zq_inputs.rng_for(8, 5)
    acc = rng.integers(-2 ** 28, 2 ** 28, size=(9, 48)).astype(np.int32)
    s_tok = zq_inputs.random_scales(rng, 9)
    s_w = zq_inputs.random_scales(rng, 3)
    bias = zq_inputs.bias(rng, 48)
    ref, _ = orc.dequant(acc, s_tok, s_w, bias)
    want = (acc.astype(np.float64) * s_tok.astype(np.float64)[:, None]
            * np.repeat(s_w.astype(np.float64), 16)[None, :] + bias.astype(np.float64)[None, :])
    assert np.allclose(ref, want, rtol=1e-15, atol=0)


def test_quantized_linear_approximates_the_fp_linear():
    """End to end on the oracle: quantize, integer GeMM, dequantize ~ x @ W^T + b.
    Ties the pieces together: a wrong scale pairing or group lookup blows the error up."""
    rng = zq_inputs.rng_for(8, 6)
    x16 = zq_inputs.activations(rng, 16, 256, n_outliers=2, outlier_scale=10.0)
    w16 = zq_inputs.weights(rng, 64, 256)
    b16 = zq_inputs.bias(rng, 64)
    xq, s_tok = orc.quant_tokenwise(x16.astype(np.float32))
    wq, s_w, _ = orc.quantize_weight_groupwise(w16, 4, 8)
    ref, _ = orc.dequant(orc.matmul_i32(xq, wq), s_tok, s_w, b16)
    exact = x16.astype(np.float64) @ w16.astype(np.float64).T + b16.astype(np.float64)
    rel = np.linalg.norm(ref - exact) / np.linalg.norm(exact)
    assert rel < 0.03
    # INT4 weights are coarser but still track
    wq4, s_w4, codes4 = orc.quantize_weight_groupwise(w16, 4, 4)
    ref4, _ = orc.dequant(orc.matmul_i32(xq, codes4), s_tok, s_w4, b16)
    rel4 = np.linalg.norm(ref4 - exact) / np.linalg.norm(exact)
    assert rel < rel4 < 0.3


def test_matmul_f16_i8_pins():
    """FP16 x INT8 product in fp64: a Python triple loop with exact rationals, numpy float64 matmul,
    integer-valued activations reduce to the int32 product, selector rows pick single weight columns,
    and the row subset equals the rows of the full result."""
    from fractions import Fraction
    rng = zq_inputs.rng_for(8, 1)
    M, N, K = 3, 5, 16
    x = (rng.standard_normal((M, K)) * 3).astype(np.float16)
    w = zq_inputs.random_codes(rng, (N, K))
    acc, absacc = orc.matmul_f16_i8(x, w)
    for m in range(M):
        for n in range(N):
            s = sum(Fraction(float(x[m, k])) * int(w[n, k]) for k in range(K))
            a = sum(abs(Fraction(float(x[m, k])) * int(w[n, k])) for k in range(K))
            assert acc[m, n] == float(s) and absacc[m, n] == float(a)
    M, N, K = 9, 48, 1040
    x = (rng.standard_normal((M, K)) * 2).astype(np.float16)
    w = zq_inputs.random_codes(rng, (N, K))
    acc, absacc = orc.matmul_f16_i8(x, w)
    want = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.abs(acc - want).max() <= 1e-9 * np.abs(absacc).max()
    assert (absacc >= np.abs(acc) - 1e-9).all()
    xi = zq_inputs.random_codes(rng, (M, K))
    acc_i, _ = orc.matmul_f16_i8(xi.astype(np.float16), w)          # |codes| <= 127 are exact in FP16
    assert np.array_equal(acc_i, orc.matmul_i32(xi, w).astype(np.float64))
    sel = np.zeros((2, K), np.float16)
    sel[0, 7] = 1.0
    sel[1, 1039] = -0.5
    acc_s, _ = orc.matmul_f16_i8(sel, w)
    assert np.array_equal(acc_s[0], w[:, 7].astype(np.float64)) and np.array_equal(acc_s[1], -0.5 * w[:, 1039])
    sub, sub_abs = orc.matmul_f16_i8(x, w, rows=[8, 0, 3])
    assert np.array_equal(sub, acc[[8, 0, 3]]) and np.array_equal(sub_abs, absacc[[8, 0, 3]])


def test_dequant_w_pins():
    acc = np.array([[2.0, -4.0] + [0.0] * 30, [1.0, 1.0] + [3.0] * 30])
    s_w = np.array([0.5, 0.25], np.float32)
    bias = np.zeros(32, np.float16)
    bias[1] = 1.0
    ref, mag = orc.dequant_w(acc, s_w, bias)
    assert ref[0, 0] == 1.0 and ref[0, 1] == -1.0 and mag[0, 1] == 3.0
    assert ref[1, 16] == 0.75 and ref[1, 31] == 0.75 and ref[1, 15] == 1.5
    ref2, _ = orc.dequant_w(acc, s_w, None)
    assert ref2[0, 1] == -2.0
