"""GPU parity on seeded random shapes through the default dispatch: whatever schedule the library
picks for a shape (streaming with or without K ranges and K splits, tiles, tiles with a K split,
untiled), the INT32 accumulators equal the oracle's bit for bit and the FP16 output is within the
tolerance, for INT8 and INT4 weights; the W8A16 call within its own tolerance."""
import numpy as np
import pytest
import torch

import zq_inputs
from helpers import assert_bit_equal, assert_out_close, dev, host

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


def _shapes(seed, count):
    rnd = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        # token counts around every boundary of the dispatcher, columns and depth up to a few thousand
        M = int(rnd.choice([1, 7, 16, 17, 33, 64, 65, 100, 128, 129, 200, 300, 520]))
        N = 16 * int(rnd.integers(1, 260))
        K = int(rnd.choice([256, 512, 1024, 2048, 4096, 4352, 8192])) if rnd.random() < 0.7 else 32 * int(rnd.integers(1, 200))
        if M * N * K > 1.2e9:
            continue
        gs = [d for d in (1, 2, 3, 4, 5, 8, 13, 16) if (N // 16) % d == 0]
        out.append((M, N, K, (N // 16) // int(rnd.choice(gs))))
    return out


SHAPES = _shapes(20220601, 36)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,N,K,g", SHAPES)
def test_default_dispatch_against_oracle(zq, orc, bits, M, N, K, g):
    nbytes = zq.gemm_workspace_bytes(M, N, K, bits)
    name = zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, bits, nbytes))
    print("random", bits, M, N, K, g, name, flush=True)
    rng = zq_inputs.rng_for(11, M + N + K + bits)
    xq = zq_inputs.random_codes(rng, (M, K))
    s_tok = zq_inputs.random_scales(rng, M, 5e-3, 0.3)
    s_w = zq_inputs.random_scales(rng, g, 1e-4, 1e-3)
    bias = zq_inputs.bias(rng, N, std=0.05)
    codes = zq_inputs.random_codes(rng, (N, K), qmax=127 if bits == 8 else 7)
    if bits == 8:
        wq = codes
    else:
        u = codes.astype(np.uint8) & 0xF
        wq = (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)
    ws = zq.new_workspace(nbytes)
    fn = zq.zq_gemm_i8_dequant if bits == 8 else zq.zq_gemm_w4a8_dequant
    out, acc, _, _ = fn(dev(xq), dev(s_tok), dev(wq), dev(s_w), dev(bias), want_acc=True, workspace=ws)
    torch.cuda.synchronize()
    acc_o = orc.matmul_i32(xq, codes)
    assert_bit_equal(host(acc), acc_o, "%s acc" % name)
    ref, mag = orc.dequant(acc_o, s_tok, s_w, bias)
    assert_out_close(host(out), ref, mag, "%s out" % name)


@pytest.mark.parametrize("M,N,K,g", SHAPES[::3])
def test_default_dispatch_w8a16(zq, orc, M, N, K, g):
    from test_gpu_gemm_a16 import _check
    print("random w8a16", M, N, K, g, flush=True)
    rng = zq_inputs.rng_for(12, M + N + K)
    x = zq_inputs.activations(rng, M, K, outlier_frac=0.01, outlier_scale=15.0)
    codes = zq_inputs.random_codes(rng, (N, K))
    s_w = zq_inputs.random_scales(rng, g, 1e-4, 1e-2)
    bias = zq_inputs.bias(rng, N)
    nbytes = zq.gemm_w8a16_workspace_bytes(M, N, K)
    ws = zq.new_workspace(nbytes)
    out = zq.zq_gemm_w8a16_dequant(dev(x), dev(codes), dev(s_w), dev(bias), workspace=ws)
    torch.cuda.synchronize()
    _check(orc, host(out), x, codes, s_w, bias, "random w8a16 %dx%dx%d" % (M, N, K))
