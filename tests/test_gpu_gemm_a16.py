"""GPU parity of the W8A16 GeMM (FP16 activations x group-wise INT8 weights, Sec. 5) against the
fp64 oracle, through the C ABI.  Accumulation is fp32 on the matrix cores, so the bar is the FP16
tolerance of the task (2e-3 of the terms' magnitude) plus the fp32 accumulation bound."""
import numpy as np
import pytest
import torch

import zq_inputs
from helpers import dev, host
from test_gpu_gemm import orc, zq  # noqa: F401 (fixtures)

pytestmark = pytest.mark.gpu


def _check(orc, out16, x, codes, s_w, bias, what, rows=None):
    K = x.shape[1]
    acc, absacc = orc.matmul_f16_i8(x, codes, rows=rows)
    ref, mag = orc.dequant_w(acc, s_w, bias)
    gs = codes.shape[0] // s_w.size
    sw_col = np.repeat(s_w.astype(np.float64), gs)[None, :]
    # one FP16 rounding of the result (4.9e-4 relative, inside the task's 2e-3), and at most one fp32
    # rounding per 16-deep matrix-core step on partial sums no larger than the sum of |products|
    tol = 2e-3 * mag + (K / 16 + 8) * 2.0 ** -24 * absacc * sw_col + 2.0 ** -25
    got = out16.astype(np.float64) if rows is None else out16[rows].astype(np.float64)
    err = np.abs(got - ref)
    assert (err <= tol).all(), "%s: %d bad, worst err %.3e at tol %.3e" % (
        what, int((err > tol).sum()), err.max(), tol[np.unravel_index(err.argmax(), err.shape)])
    # the accumulation term must not be what makes the test pass: typical error is far below it
    assert np.median(err / np.maximum(mag, 1e-30)) < 5e-4, what


SHAPES = [
    # (M, N, K, groups): the untiled schedule (ragged K, M > 128) ...
    (1, 16, 16, 1), (17, 768, 784, 48), (129, 96, 1024, 2), (70, 272, 208, 17),
    # ... the streaming schedule, one to four token tiles, uneven strips ...
    (1, 64, 256, 4), (8, 6144, 2048, 128), (33, 144, 1792, 9), (64, 1024, 1536, 64), (16, 33040, 512, 5),
    (50, 16, 256, 1),
    # ... the tiled schedules (128x128 and 256x256 tiles, ragged edges) ...
    (300, 400, 384, 25), (515, 1024, 1024, 64), (129, 272, 2048, 17), (2500, 4112, 512, 257),
    (515, 1024, 400, 64), (300, 1040, 1008, 65),       # K not a multiple of the stage depth
    (2300, 7152, 336, 3),                              # 256x256 tiles (one round of 252), ragged in M, N and K
    # ... and with a K split
    (32, 2048, 8192, 128), (7, 528, 24576, 11), (64, 4112, 16384, 1), (1, 2048, 8192, 128),
    # above 128 tokens with few tiles and a long K: the tiled schedule splits K (fp32 partials, second kernel)
    (130, 1024, 4096, 64), (300, 400, 2048, 25), (256, 2064, 2000, 3), (129, 272, 8192, 17),
    # 65 to 128 tokens: two streaming launches over row halves (second half ragged, one row, full), also with a K split
    (65, 1024, 1536, 64), (100, 6144, 2048, 128), (128, 2064, 512, 3), (90, 2048, 8192, 128), (128, 528, 24576, 11),
]


@pytest.mark.parametrize("M,N,K,g", SHAPES)
def test_w8a16_against_oracle(zq, orc, M, N, K, g):
    print("w8a16", M, N, K, g, flush=True)
    rng = zq_inputs.rng_for(9, M + N + K)
    x = zq_inputs.activations(rng, M, K, outlier_frac=0.01, outlier_scale=15.0)
    codes = zq_inputs.random_codes(rng, (N, K))
    s_w = zq_inputs.random_scales(rng, g, 1e-4, 1e-2)
    bias = zq_inputs.bias(rng, N)
    nbytes = zq.gemm_w8a16_workspace_bytes(M, N, K)
    ws = zq.new_workspace(nbytes)
    out = zq.zq_gemm_w8a16_dequant(dev(x), dev(codes), dev(s_w), dev(bias), workspace=ws)
    out2 = zq.zq_gemm_w8a16_dequant(dev(x), dev(codes), dev(s_w), dev(bias), workspace=ws)
    torch.cuda.synchronize()
    _check(orc, host(out), x, codes, s_w, bias, "w8a16 %dx%dx%d" % (M, N, K))
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16)), "result depends on arrival order"
    # without a workspace (no K split) and without bias
    out3 = zq.zq_gemm_w8a16_dequant(dev(x), dev(codes), dev(s_w), None)
    torch.cuda.synchronize()
    _check(orc, host(out3), x, codes, s_w, None, "w8a16 no ws/bias %dx%dx%d" % (M, N, K))


def test_w8a16_integer_inputs_are_exact(zq, orc):
    """Integer-valued activations make every partial sum an integer below 2^24: fp32 accumulation is
    exact, so the result equals the INT8 x INT8 product dequantized with unit token scales."""
    rng = zq_inputs.rng_for(9, 4)
    M, N, K, g = 24, 256, 768, 16
    xq = zq_inputs.random_codes(rng, (M, K))
    codes = zq_inputs.random_codes(rng, (N, K))
    s_w = np.full(g, 2.0 ** -12, np.float32)
    out = zq.zq_gemm_w8a16_dequant(dev(xq.astype(np.float16)), dev(codes), dev(s_w), None)
    torch.cuda.synchronize()
    acc = orc.matmul_i32(xq, codes).astype(np.float64)
    assert np.abs(acc).max() < 2 ** 24
    want = (acc * 2.0 ** -12).astype(np.float16)          # one rounding, as the kernel does
    assert np.array_equal(host(out).view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("name,M", [("c5_qkv", 64), ("c4_qkv", 16), ("c4_qkv", 128), ("c3_qkv", 1), ("c3_qkv", 2048), ("c4_qkv", 4096)])
def test_w8a16_full_size_sampled_rows(zq, orc, name, M):
    """QKV linears at workload size in the launch configuration the benchmark times; sampled rows."""
    K, N, g, bits = zq_inputs.LINEARS[name]
    gen = torch.Generator(device="cuda").manual_seed(99)
    x = (torch.randn((M, K), generator=gen, device="cuda") *
         torch.exp(torch.empty((M, 1), device="cuda").uniform_(-0.7, 0.7, generator=gen))).half()
    codes = torch.randint(-127, 128, (N, K), generator=gen, device="cuda", dtype=torch.int8)
    s_w = (torch.rand(g, generator=gen, device="cuda") * 1e-3 + 1e-4)
    bias = (torch.randn(N, generator=gen, device="cuda") * 0.01).half()
    nbytes = zq.gemm_w8a16_workspace_bytes(M, N, K)
    ws = zq.new_workspace(nbytes)
    out = zq.zq_gemm_w8a16_dequant(x, codes, s_w, bias, workspace=ws)
    torch.cuda.synchronize()
    rows = sorted(set([0, M - 1, M // 2, min(M - 1, 15), min(M - 1, 16), min(M - 1, 255), min(M - 1, 256)]))
    _check(orc, host(out), host(x), host(codes), host(s_w), host(bias), "w8a16 %s M=%d" % (name, M), rows=rows)
