"""GPU parity: group-wise weight quantization and the fused LayerNorm / GeLU
front-ends against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import zq_inputs
from helpers import assert_bit_equal, check_fused_codes, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zq():
    import paper_2206_01861_amd as lib
    lib.lib()
    return lib


@pytest.fixture(scope="module")
def orc():
    from oracle import zq_oracle
    return zq_oracle


# ---------------------------------------------------------------- weights ----
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("N,K,g", [
    (768, 768, 48),        # BERT-base, 16 rows per group
    (4096, 1024, 64),      # BERT-large FFC1
    (1024, 4096, 64),      # BERT-large FFC2
    (6144, 2048, 128),     # GPT-3 1.3B QKV, 48 rows per group
    (16, 32, 1),           # smallest legal matrix
    (96, 4128, 2),         # K not a multiple of the vector stride
    (2048, 160, 128),
])
def test_weight_quant_bit_exact(zq, orc, bits, N, K, g):
    print("weight quant", bits, N, K, g, flush=True)
    rng = zq_inputs.rng_for(1, N + K + bits)
    w = zq_inputs.weights(rng, N, K)
    if g > 2:
        w[(N // g):(2 * N // g)] = 0          # an all-zero group: codes 0, scale 0
    wq_o, s_o, _ = orc.quantize_weight_groupwise(w, g, bits)
    wq, s_w = zq.zq_quantize_weight_groupwise(dev(w), g, bits)
    torch.cuda.synchronize()
    assert_bit_equal(host(s_w), s_o, "s_w")
    assert_bit_equal(host(wq), wq_o, "wq")


def test_weight_quant_fp16_extremes(zq, orc):
    # subnormal-only group, a group holding the largest fp16, and exact ties
    N, K, g = 48, 64, 3
    w = np.zeros((N, K), np.float16)
    w[0:16] = np.float16(6e-8) * np.arange(K, dtype=np.float16)[None, :]
    w[16:32] = np.linspace(-65504, 65504, 16 * K).astype(np.float16).reshape(16, K)
    w[32:48] = (np.arange(16 * K) % 255 - 127).astype(np.float16).reshape(16, K) * np.float16(0.5)
    for bits in (8, 4):
        wq_o, s_o, _ = orc.quantize_weight_groupwise(w, g, bits)
        wq, s_w = zq.zq_quantize_weight_groupwise(dev(w), g, bits)
        assert_bit_equal(host(s_w), s_o, "s_w")
        assert_bit_equal(host(wq), wq_o, "wq")


# ------------------------------------------------------------ front-ends ----
ROW_SHAPES = [(1, 768), (7, 768), (33, 1024), (129, 2048), (5, 4096), (4, 6144), (3, 8192),
              (2, 16384), (2, 24576), (9, 16), (6, 1040), (2, 32768)]


@pytest.mark.parametrize("M,K", ROW_SHAPES)
def test_layernorm_quant(zq, orc, M, K):
    print("layernorm", M, K, flush=True)
    rng = zq_inputs.rng_for(2, M + K)
    x = zq_inputs.activations(rng, M, K, outlier_frac=0.01, outlier_scale=15.0, token_spread=True)
    gamma, beta = zq_inputs.layernorm_params(rng, K)
    xq, s_tok, y = zq.zq_layernorm_quant_tokenwise(dev(x), dev(gamma), dev(beta), 1e-5, y_dtype=torch.float32)
    torch.cuda.synchronize()
    xq, s_tok, y = host(xq), host(s_tok), host(y)
    # the quantizer itself, on exactly the fp32 values the kernel quantized: bit-exact
    xq_o, s_o = orc.quant_tokenwise(y)
    assert_bit_equal(s_tok, s_o, "s_tok")
    assert_bit_equal(xq, xq_o, "xq")
    # the fused chain against the all-fp64 LayerNorm
    y64, _ = orc.layernorm(x, gamma, beta, 1e-5)
    n_mis = check_fused_codes(xq, s_tok, y, y64, "layernorm %dx%d" % (M, K))
    assert n_mis <= max(4, int(1e-3 * M * K))


def test_layernorm_options(zq, orc):
    rng = zq_inputs.rng_for(2, 999)
    M, K = 12, 1024
    x = zq_inputs.activations(rng, M, K, n_outliers=4, outlier_scale=20.0)
    x[5] = np.float16(1.25)          # constant row: zero variance, y = beta
    gamma, beta = zq_inputs.layernorm_params(rng, K)
    # no beta, fp16 tap, other eps
    xq, s_tok, y16 = zq.zq_layernorm_quant_tokenwise(dev(x), dev(gamma), None, 1e-12, y_dtype=torch.float16)
    y64, _ = orc.layernorm(x, gamma, None, 1e-12)
    check_fused_codes(host(xq), host(s_tok), None, y64, "layernorm no beta")
    assert np.abs(host(y16).astype(np.float64) - y64).max() <= 1e-3 * np.abs(y64).max()
    assert host(s_tok)[5] == 0 and not host(xq)[5].any()      # zero row: codes 0, scale 0
    # no tap at all gives the same codes as with the tap
    xq2, s2, none = zq.zq_layernorm_quant_tokenwise(dev(x), dev(gamma), None, 1e-12)
    assert none is None
    assert torch.equal(xq2, xq) and torch.equal(s2, s_tok)


@pytest.mark.parametrize("approx", [False, True])
@pytest.mark.parametrize("M,N", [(1, 4096), (7, 3072), (33, 8192), (3, 16384), (2, 24576), (130, 768)])
def test_gelu_quant(zq, orc, approx, M, N):
    print("gelu", approx, M, N, flush=True)
    rng = zq_inputs.rng_for(3, M + N)
    h = (zq_inputs.activations(rng, M, N, outlier_frac=0.01, outlier_scale=6.0).astype(np.float32) * 1.5).astype(np.float16)
    bias = zq_inputs.bias(rng, N, std=0.2)
    xq, s_tok, y = zq.zq_gelu_quant_tokenwise(dev(h), dev(bias), approx_tanh=approx, y_dtype=torch.float32)
    torch.cuda.synchronize()
    xq, s_tok, y = host(xq), host(s_tok), host(y)
    xq_o, s_o = orc.quant_tokenwise(y)
    assert_bit_equal(s_tok, s_o, "s_tok")
    assert_bit_equal(xq, xq_o, "xq")
    y64, _ = orc.gelu(h, bias, approx_tanh=approx)
    n_mis = check_fused_codes(xq, s_tok, y, y64, "gelu %dx%d" % (M, N))
    assert n_mis <= max(4, int(1e-3 * M * N))
    # bias is optional
    xq_nb, s_nb, y_nb = zq.zq_gelu_quant_tokenwise(dev(h), None, approx_tanh=approx, y_dtype=torch.float32)
    y64_nb, _ = orc.gelu(h, None, approx_tanh=approx)
    check_fused_codes(host(xq_nb), host(s_nb), host(y_nb), y64_nb, "gelu no bias")


@pytest.mark.parametrize("with_bias", [False, True])
def test_gelu_of_every_fp16_input(zq, orc, with_bias):
    """The kernel's GeLU (erf form) over all 63488 finite FP16 inputs, alone and with a bias that
    moves them off the FP16 grid: within 2.5e-7 + 2e-6 |y| of the fp64 value (the kernel's
    approximation is good to 1.2e-7 absolute; the relative term covers fp32 rounding of large values).
    Subnormal inputs and both zeros included."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    h = bits.view(np.float16)
    h = h[np.isfinite(h)]
    pad = (-h.size) % 4096
    h = np.concatenate([h, np.zeros(pad, np.float16)]).reshape(-1, 4096)
    bias = None
    if with_bias:
        bias = zq_inputs.bias(zq_inputs.rng_for(3, 4242), 4096, std=0.37)
    _, _, y = zq.zq_gelu_quant_tokenwise(dev(h), None if bias is None else dev(bias), y_dtype=torch.float32)
    y = host(y).astype(np.float64)
    y64, _ = orc.gelu(h, bias)
    err = np.abs(y - y64)
    tol = 2.5e-7 + 2e-6 * np.abs(y64)
    assert (err <= tol).all(), "worst %.3e at h=%r" % ((err - tol).max(), h.ravel()[(err - tol).argmax()])


@pytest.mark.parametrize("M,K", [(1, 16), (5, 768), (64, 4096), (3, 32768), (130, 1040)])
def test_standalone_tokenwise_quantizer(zq, orc, M, K):
    """The quantization operator on its own (Sec. 4.3): bit-exact against the oracle, zero rows included."""
    rng = zq_inputs.rng_for(3, 900 + M + K)
    x = zq_inputs.activations(rng, M, K, outlier_frac=0.01, outlier_scale=15.0)
    if M > 2:
        x[2] = 0
    xq, s = zq.zq_quantize_tokenwise(dev(x))
    torch.cuda.synchronize()
    q_o, s_o = orc.quant_tokenwise(x.astype(np.float32))
    assert_bit_equal(host(s), s_o, "s_tok")
    assert_bit_equal(host(xq), q_o, "xq")


@pytest.mark.parametrize("M,N,g", [(1, 16, 1), (37, 256, 16), (300, 4096, 64), (5, 48, 3)])
def test_standalone_dequantizer(zq, orc, M, N, g):
    """The dequantization epilogue as its own kernel (App. D): within the FP16 tolerance of the fp64
    reference, and within one FP16 step of what the GeMM writes for the same accumulators (a fused
    multiply-add in one epilogue and a separate multiply and add in another may round differently)."""
    from helpers import assert_out_close
    rng = zq_inputs.rng_for(3, 950 + M + N)
    acc = rng.integers(-2 ** 30, 2 ** 30, size=(M, N), dtype=np.int64).astype(np.int32)
    acc[0, :4] = [0, 1, -1, 2 ** 31 - 1]
    s_tok = zq_inputs.random_scales(rng, M, 1e-7, 1e-5)
    s_w = zq_inputs.random_scales(rng, g, 1e-4, 1e-2)
    bias = zq_inputs.bias(rng, N)
    for b in (bias, None):
        out = zq.zq_dequantize_acc(dev(acc), dev(s_tok), dev(s_w), None if b is None else dev(b))
        torch.cuda.synchronize()
        ref, mag = orc.dequant(acc, s_tok, s_w, b)
        assert_out_close(host(out), ref, mag, "dequant %dx%d" % (M, N))
    # agrees with the fused epilogue
    K = 256
    xq = zq_inputs.random_codes(rng, (M, K))
    wq = zq_inputs.random_codes(rng, (N, K))
    o, a, _, _ = zq.zq_gemm_i8_dequant(dev(xq), dev(s_tok), dev(wq), dev(s_w), dev(bias), want_acc=True)
    o2 = zq.zq_dequantize_acc(a, dev(s_tok), dev(s_w), dev(bias))
    torch.cuda.synchronize()
    d = (o.float() - o2.float()).abs()
    assert bool((d <= o.float().abs() * 2.0 ** -10 + 2.0 ** -24).all())


def test_kernels_reproduce_the_frozen_small_case(zq):
    """The stored oracle outputs of tests/golden/quantizer_small.txt, reproduced by the HIP kernels bit for bit."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "quantizer_small.txt")
    rec = dict(line.split(" ", 1) for line in open(path).read().splitlines() if not line.startswith("#"))
    w = np.frombuffer(bytes.fromhex(rec["w_fp16_hex"]), np.float16).reshape(32, 32)
    x = np.frombuffer(bytes.fromhex(rec["x_fp16_hex"]), np.float16).reshape(4, 32)
    for bits in (8, 4):
        wq, s_w = zq.zq_quantize_weight_groupwise(dev(w.copy()), 2, bits)
        torch.cuda.synchronize()
        assert host(wq).view(np.uint8).tobytes().hex() == rec["w%d_packed_hex" % bits]
        assert host(s_w).view(np.uint32).tobytes().hex() == rec["w%d_scale_hex" % bits]
    xq, s_tok = zq.zq_quantize_tokenwise(dev(x.copy()))
    wq8, s_w8 = zq.zq_quantize_weight_groupwise(dev(w.copy()), 2, 8)
    _, acc, _, _ = zq.zq_gemm_i8_dequant(xq, s_tok, wq8, s_w8, None, want_acc=True)
    torch.cuda.synchronize()
    assert host(xq).view(np.uint8).tobytes().hex() == rec["x_codes_hex"]
    assert host(s_tok).view(np.uint32).tobytes().hex() == rec["x_scale_hex"]
    assert " ".join(str(int(v)) for v in host(acc).ravel()) == rec["acc_i32"]


def test_front_ends_at_workload_size(zq, orc):
    """LayerNorm+quant and GeLU+quant on the full 4096-token BERT-large tensors the benchmark times:
    codes and scales bit-exact given the fp32 tap for every element, fused values against the fp64
    chain on sampled rows."""
    rng = zq_inputs.rng_for(2, 11)
    M, H, F = 4096, 1024, 4096
    x = zq_inputs.config_activations("c2", rng, M, H)
    gamma, beta = zq_inputs.layernorm_params(rng, H)
    xq, s_tok, y = zq.zq_layernorm_quant_tokenwise(dev(x), dev(gamma), dev(beta), 1e-5, y_dtype=torch.float32)
    torch.cuda.synchronize()
    q_o, s_o = orc.quant_tokenwise(host(y))
    assert_bit_equal(host(s_tok), s_o, "LN s_tok")
    assert_bit_equal(host(xq), q_o, "LN codes")
    rows = [0, 1, 255, 256, 2047, 4095]
    y64, _ = orc.layernorm(x[rows], gamma, beta, 1e-5)
    check_fused_codes(host(xq)[rows], host(s_tok)[rows], host(y)[rows], y64, "LN 4096x1024")

    h = (zq_inputs.activations(rng, M, F, outlier_frac=0.01, outlier_scale=6.0).astype(np.float32) * 1.5).astype(np.float16)
    hq, s2, y2 = zq.zq_gelu_quant_tokenwise(dev(h), None, y_dtype=torch.float32)
    torch.cuda.synchronize()
    q_o, s_o = orc.quant_tokenwise(host(y2))
    assert_bit_equal(host(s2), s_o, "GeLU s_tok")
    assert_bit_equal(host(hq), q_o, "GeLU codes")
    g64, _ = orc.gelu(h[rows], None)
    check_fused_codes(host(hq)[rows], host(s2)[rows], host(y2)[rows], g64, "GeLU 4096x4096")
