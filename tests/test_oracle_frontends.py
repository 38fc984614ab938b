"""Pins for the oracle's LayerNorm and bias+GeLU (the operators the token-wise
quantizer is fused behind, Sec. 4.3 / App. D).  The paper names the operators
without formulas; they are pinned to torch's float64 library routines and to
closed forms."""
import math

import numpy as np
import torch

import zq_inputs
from oracle import zq_oracle as orc


def test_layernorm_matches_torch_float64():
    rng = zq_inputs.rng_for(7, 1)
    x = zq_inputs.activations(rng, 13, 768, n_outliers=4, outlier_scale=20.0)
    g, b = zq_inputs.layernorm_params(rng, 768)
    for eps in (1e-5, 1e-12):
        y64, y32 = orc.layernorm(x, g, b, eps)
        want = torch.nn.functional.layer_norm(
            torch.from_numpy(x.astype(np.float64)), (768,),
            torch.from_numpy(g.astype(np.float64)), torch.from_numpy(b.astype(np.float64)), eps).numpy()
        assert np.abs(y64 - want).max() <= 1e-12 * max(1.0, np.abs(want).max())
        assert np.array_equal(y32, y64.astype(np.float32))
    y64n, _ = orc.layernorm(x, g, None, 1e-5)
    want = torch.nn.functional.layer_norm(
        torch.from_numpy(x.astype(np.float64)), (768,),
        torch.from_numpy(g.astype(np.float64)), None, 1e-5).numpy()
    assert np.abs(y64n - want).max() <= 1e-12 * np.abs(want).max()


def test_layernorm_closed_forms():
    # constant row -> zero deviation -> y = beta
    K = 32
    x = np.full((1, K), 3.0, np.float16)
    g = np.full(K, 2.0, np.float16)
    b = np.arange(K).astype(np.float16)
    y64, _ = orc.layernorm(x, g, b, 1e-5)
    assert np.array_equal(y64[0], b.astype(np.float64))
    # row (+1,-1,...) has mean 0, variance 1: y = x*gamma/sqrt(1+eps)
    x = np.tile(np.array([1.0, -1.0], np.float16), K // 2)[None, :]
    y64, _ = orc.layernorm(x, g, None, 0.25)
    assert np.allclose(y64[0], x[0].astype(np.float64) * 2.0 / math.sqrt(1.25), rtol=1e-15)


def test_gelu_matches_torch_float64_both_forms():
    rng = zq_inputs.rng_for(7, 2)
    h = (4 * rng.standard_normal((11, 96))).astype(np.float16)
    bias = zq_inputs.bias(rng, 96, std=0.5)
    u = torch.from_numpy(h.astype(np.float64) + bias.astype(np.float64)[None, :])
    y64, y32 = orc.gelu(h, bias, approx_tanh=False)
    want = torch.nn.functional.gelu(u).numpy()
    assert np.abs(y64 - want).max() <= 1e-13
    assert np.array_equal(y32, y64.astype(np.float32))
    y64t, _ = orc.gelu(h, bias, approx_tanh=True)
    want_t = torch.nn.functional.gelu(u, approximate="tanh").numpy()
    assert np.abs(y64t - want_t).max() <= 1e-13
    assert np.abs(y64t - y64).max() > 1e-5      # the two forms are distinguishable
    y64n, _ = orc.gelu(h, None)
    assert np.abs(y64n - torch.nn.functional.gelu(torch.from_numpy(h.astype(np.float64))).numpy()).max() <= 1e-13


def test_gelu_closed_forms():
    h = np.array([[0.0, 1.0, -1.0, 8.0, -8.0]], np.float16)
    y64, _ = orc.gelu(h, None)
    phi1 = 0.5 * (1 + math.erf(1 / math.sqrt(2)))
    assert y64[0, 0] == 0.0
    assert abs(y64[0, 1] - phi1) < 1e-15
    assert abs(y64[0, 2] + (1 - phi1)) < 1e-15
    assert abs(y64[0, 3] - 8.0) < 1e-12 and abs(y64[0, 4]) < 1e-12


def test_gelu_f64_pins():
    """GeLU on fp64 inputs: the library's float64 GeLU, the identity gelu(x) - gelu(-x) = x
    (Phi(x) + Phi(-x) = 1; tanh is odd), closed values, and agreement with the FP16-input routine."""
    rng = zq_inputs.rng_for(7, 5)
    u = 5 * rng.standard_normal((7, 33))
    for approx in (False, True):
        y = orc.gelu_f64(u, approx)
        want = torch.nn.functional.gelu(torch.from_numpy(u), approximate="tanh" if approx else "none").numpy()
        assert np.abs(y - want).max() <= 1e-13
        assert np.abs(y - orc.gelu_f64(-u, approx) - u).max() <= 1e-13
    phi1 = 0.5 * (1 + math.erf(1 / math.sqrt(2)))
    y = orc.gelu_f64(np.array([0.0, 1.0, -1.0, 40.0, -40.0]))
    assert y[0] == 0.0 and abs(y[1] - phi1) < 1e-15 and abs(y[2] + (1 - phi1)) < 1e-15
    assert y[3] == 40.0 and y[4] == 0.0
    h = (4 * rng.standard_normal((5, 48))).astype(np.float16)
    y64, _ = orc.gelu(h, None)
    assert np.array_equal(orc.gelu_f64(h.astype(np.float64)), y64)
    assert np.abs(orc.gelu_f64(u, True) - orc.gelu_f64(u, False)).max() > 1e-5
