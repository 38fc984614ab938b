"""GPU parity: the INT8 / W4A8 GeMM with its dequantization epilogue against
the CPU oracle, for every schedule, through the C ABI.  Integer results are
compared bit for bit, FP16 outputs within 2e-3 of the fp64 reference."""
import numpy as np
import pytest
import torch

import zq_inputs
from helpers import assert_bit_equal, assert_out_close, dev, freivalds_gpu, host

pytestmark = pytest.mark.gpu

SIMPLE, TILE128, TILE256, SKINNY, SKINNY_SPLITK, TILE256X128, TILE256X192, TILE_SPLITK = range(8)


@pytest.fixture(scope="module")
def zq():
    import paper_2206_01861_amd as lib
    lib.lib()
    return lib


@pytest.fixture(scope="module")
def orc():
    from oracle import zq_oracle
    return zq_oracle


def _case(rng, M, N, K, g, bits):
    xq = zq_inputs.random_codes(rng, (M, K))
    xq[:, 0] = 127
    s_tok = zq_inputs.random_scales(rng, M, 5e-3, 0.3)
    s_w = zq_inputs.random_scales(rng, g, 1e-4, 1e-3)
    bias = zq_inputs.bias(rng, N, std=0.05)
    codes = zq_inputs.random_codes(rng, (N, K), qmax=127 if bits == 8 else 7)
    if bits == 8:
        wq = codes
    else:
        u = codes.astype(np.uint8) & 0xF
        wq = (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)
    return xq, s_tok, s_w, bias, codes, wq


def _run(zq, bits, variant, xq, s_tok, wq, s_w, bias, workspace=None, requant=False):
    fn = zq.zq_gemm_i8_dequant if bits == 8 else zq.zq_gemm_w4a8_dequant
    prev = zq.force_gemm_variant(variant)
    try:
        res = fn(dev(xq), dev(s_tok), dev(wq), dev(s_w), None if bias is None else dev(bias),
                 want_acc=True, requant=requant, workspace=workspace)
        torch.cuda.synchronize()
    finally:
        zq.force_gemm_variant(prev)
    return res


def _check(orc, res, xq, s_tok, codes, s_w, bias, what):
    out, acc = host(res[0]), host(res[1])
    acc_o = orc.matmul_i32(xq, codes)
    assert_bit_equal(acc, acc_o, what + " acc")
    ref, mag = orc.dequant(acc_o, s_tok, s_w, bias)
    assert_out_close(out, ref, mag, what + " out")


# (variant, M, N, K, groups): several tiles in each direction plus ragged tails
# Every shape runs with INT8 and with INT4 weights.  With INT4 weights the TILE128 and TILE_SPLITK cases take the kernel that keeps
# the nibbles packed in LDS and unpacks them after the fragment read (its k steps visit K in a permuted order, so
# the K tails of 32, 96, 544, 800 and 4000 below are the cases that matter for it); the other tiled cases unpack on
# the way into LDS.
SHAPES = [
    (SIMPLE, 1, 16, 16, 1), (SIMPLE, 7, 48, 80, 3), (SIMPLE, 17, 768, 784, 48), (SIMPLE, 129, 96, 1024, 2),
    (TILE128, 128, 768, 768, 48), (TILE128, 129, 272, 256, 17), (TILE128, 300, 400, 384, 25),
    (TILE128, 1, 16, 128, 1), (TILE128, 515, 1024, 1024, 64),
    # more 128x128 tiles than compute units (21 x 21, ragged in M, N and K): the ring refills many times and
    # later tiles start as earlier ones leave
    (TILE128, 2600, 2576, 544, 161), (TILE128, 2600, 2576, 1024, 161),
    (TILE256, 256, 256, 128, 16), (TILE256, 300, 528, 512, 33), (TILE256, 1030, 768, 256, 48),
    (TILE256, 17, 16, 384, 1),
    # K that is not a multiple of the stage depth: the last stage is zero filled
    (TILE128, 129, 272, 800, 17), (TILE256, 300, 528, 1056, 33), (TILE256X128, 300, 400, 96, 25), (TILE128, 17, 768, 32, 48),
    (TILE256, 70, 64, 4000, 4),
    (TILE256X128, 256, 128, 128, 8), (TILE256X128, 300, 400, 512, 25), (TILE256X128, 1030, 272, 256, 17),
    (TILE256X128, 17, 16, 384, 1), (TILE256X128, 512, 1024, 1024, 64),
    # 256 x 192 tiles: whole and ragged in both directions, ragged K, a single tile
    (TILE256X192, 256, 192, 128, 12), (TILE256X192, 300, 400, 512, 25), (TILE256X192, 1030, 768, 256, 48),
    (TILE256X192, 17, 16, 384, 1), (TILE256X192, 515, 1200, 1056, 75), (TILE256X192, 2048, 6144, 128, 128),
    (SKINNY, 1, 64, 256, 4), (SKINNY, 3, 128, 768, 8), (SKINNY, 1, 2048, 2048, 128), (SKINNY, 8, 6144, 2048, 128),
    (SKINNY, 16, 208, 1280, 13), (SKINNY, 17, 80, 512, 5), (SKINNY, 32, 2048, 2048, 128),
    (SKINNY, 33, 144, 1792, 9), (SKINNY, 64, 1024, 1536, 64), (SKINNY, 50, 16, 256, 1),
    # five to eight token tiles per consumer
    (SKINNY, 65, 256, 512, 16), (SKINNY, 100, 768, 768, 48), (SKINNY, 128, 2048, 2048, 128), (SKINNY, 113, 144, 1792, 9),
    # strips dealt unevenly over the row blocks, up to eight consumer waves per workgroup
    (SKINNY, 64, 18432, 1024, 128), (SKINNY, 16, 33040, 512, 5), (SKINNY, 9, 4112, 768, 1),
    # deep K without a split: two K ranges per strip for INT8 weights (even and odd stage counts, uneven
    # strips per row block, one to four strips per workgroup)
    (SKINNY, 1, 2048, 4096, 128), (SKINNY, 32, 1040, 4352, 65), (SKINNY, 17, 4112, 8192, 1), (SKINNY, 5, 80, 6400, 5),
    (SKINNY, 16, 12288, 4096, 96), (SKINNY, 9, 10000, 4864, 25),
    # 128x128 tiles with K split over workgroups and the epilogue in a second kernel: ragged in M, N and K,
    # two to eight splits, uneven stage counts per split, at most 128 tokens where K is no multiple of 256
    (TILE_SPLITK, 130, 1024, 4096, 64), (TILE_SPLITK, 300, 400, 2048, 25), (TILE_SPLITK, 129, 272, 4000, 17),
    (TILE_SPLITK, 200, 2064, 4096, 3), (TILE_SPLITK, 64, 528, 1920, 11), (TILE_SPLITK, 256, 1040, 3200, 65),
    # K split 3- to 12-fold, with ragged strip counts
    (SKINNY_SPLITK, 1, 2048, 8192, 128), (SKINNY_SPLITK, 8, 256, 4096, 16), (SKINNY_SPLITK, 32, 2048, 8192, 128),
    (SKINNY_SPLITK, 64, 1024, 6144, 64), (SKINNY_SPLITK, 13, 80, 2304, 5), (SKINNY_SPLITK, 33, 2064, 8192, 3),
    (SKINNY_SPLITK, 20, 1040, 12288, 65), (SKINNY_SPLITK, 7, 528, 24576, 11), (SKINNY_SPLITK, 64, 4112, 16384, 1),
    (SKINNY_SPLITK, 16, 4096, 16384, 256), (SKINNY_SPLITK, 128, 2048, 8192, 128), (SKINNY_SPLITK, 90, 1040, 12288, 65),
]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("variant,M,N,K,g", SHAPES)
def test_gemm_against_oracle(zq, orc, bits, variant, M, N, K, g):
    print("gemm", zq.gemm_variant_name(variant), bits, M, N, K, g, flush=True)
    if bits == 4 and K % 32:
        pytest.skip("INT4 needs K % 32 == 0")
    if variant in (SKINNY, SKINNY_SPLITK) and K % 256:
        pytest.skip("the streaming schedule steps K by 256")
    rng = zq_inputs.rng_for(4, variant * 1000 + M + N + K + bits)
    xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, bits)
    ws = None
    if variant in (SKINNY_SPLITK, TILE_SPLITK):
        nbytes = zq.gemm_workspace_bytes(M, N, K, bits)
        if nbytes == 0:
            pytest.skip("shape does not split")
        ws = zq.new_workspace(nbytes)
    if variant == SKINNY and bits == 8 and M <= 32 and K >= 4096:
        assert zq.gemm_stream_k_ranges(M, N, K, bits, 0) == 2
    res = _run(zq, bits, variant, xq, s_tok, wq, s_w, bias, workspace=ws)
    _check(orc, res, xq, s_tok, codes, s_w, bias, "%s %d-bit %dx%dx%d" % (zq.gemm_variant_name(variant), bits, M, N, K))


def test_no_bias_and_extreme_codes(zq, orc):
    # all codes at +-127 with K at the largest workload value: |acc| = 127*127*K, no wrap
    M, N, K, g = 20, 32, 24576, 2
    xq = np.full((M, K), 127, np.int8)
    wq = np.full((N, K), 127, np.int8)
    wq[1::2] = -127
    s_tok = np.full(M, 1e-3, np.float32)
    s_w = np.full(g, 1e-4, np.float32)
    for variant in (SIMPLE, TILE128, TILE256, TILE256X128, TILE256X192, SKINNY):
        res = _run(zq, 8, variant, xq, s_tok, wq, s_w, None)
        acc = host(res[1])
        assert (acc[:, 0::2] == 16129 * K).all() and (acc[:, 1::2] == -16129 * K).all()
        _check(orc, res, xq, s_tok, wq, s_w, None, "extreme")


def test_largest_k_fills_the_accumulator(zq, orc):
    """K at the largest accepted values with every product at +-127*127: the INT32 accumulator ends
    within 0.01 % of its range and must not wrap in any schedule."""
    M, N, g = 3, 32, 2
    for K, variants in ((133136, (SIMPLE, TILE128, TILE256, TILE256X128, TILE256X192)),    # largest K the ABI takes (K % 16 == 0)
                        (133120, (SIMPLE, TILE128, TILE256, TILE256X128, TILE256X192, SKINNY, SKINNY_SPLITK))):
        xq = np.full((M, K), 127, np.int8)
        xq[1] = -127
        wq = np.full((N, K), 127, np.int8)
        wq[1::2] = -127
        s_tok = np.full(M, 1e-4, np.float32)
        s_w = np.full(g, 1e-5, np.float32)
        want = np.outer(np.array([1, -1, 1], np.int64), np.where(np.arange(N) % 2 == 0, 1, -1)) * (16129 * K)
        assert np.abs(want).max() < 2 ** 31
        for variant in variants:
            nbytes = zq.gemm_workspace_bytes(M, N, K, 8)
            ws = zq.new_workspace(nbytes)
            res = _run(zq, 8, variant, xq, s_tok, wq, s_w, None, workspace=ws)
            assert np.array_equal(host(res[1]).astype(np.int64), want), (K, variant)
            ref, mag = orc.dequant(want.astype(np.int32), s_tok, s_w, None)
            assert_out_close(host(res[0]), ref, mag, "largest K %d variant %d" % (K, variant))


def test_requant_epilogue(zq, orc):
    rng = zq_inputs.rng_for(4, 77)
    M, N, K, g = 37, 256, 512, 16
    xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, 8)
    out, acc, out_q, out_s = _run(zq, 8, -1, xq, s_tok, wq, s_w, bias, requant=True)
    # token-wise quantizer over the FP16 tensor the GeMM wrote: bit-exact
    q_o, s_o = orc.quant_tokenwise(host(out).astype(np.float32))
    assert_bit_equal(host(out_s), s_o, "out_s_tok")
    assert_bit_equal(host(out_q), q_o, "out_q")


def test_dispatch_and_determinism(zq, orc):
    rng = zq_inputs.rng_for(4, 78)
    for (M, N, K, g) in [(128, 768, 768, 48), (8, 2048, 2048, 128), (200, 512, 144, 32), (64, 8192, 784, 64),
                         (100, 4096, 2048, 64)]:
        xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, 8)
        nbytes = zq.gemm_workspace_bytes(M, N, K, 8)
        ws = zq.new_workspace(nbytes)
        r1 = _run(zq, 8, -1, xq, s_tok, wq, s_w, bias, workspace=ws)
        r2 = _run(zq, 8, -1, xq, s_tok, wq, s_w, bias, workspace=ws)
        _check(orc, r1, xq, s_tok, codes, s_w, bias, "auto %dx%dx%d" % (M, N, K))
        assert torch.equal(r1[0], r2[0]) and torch.equal(r1[1], r2[1])


def test_quantized_linear_end_to_end(zq, orc):
    """LayerNorm+quant -> GeMM -> GeLU+quant -> GeMM on BERT-large FFC shapes (fewer tokens),
    every stage checked against the oracle fed with the previous GPU stage."""
    rng = zq_inputs.rng_for(2, 5)
    M, H, F, g = 256, 1024, 4096, 64
    x = zq_inputs.config_activations("c2", rng, M, H)
    gamma, beta = zq_inputs.layernorm_params(rng, H)
    w1, b1 = zq_inputs.weights(rng, F, H), zq_inputs.bias(rng, F)
    w2, b2 = zq_inputs.weights(rng, H, F), zq_inputs.bias(rng, H)
    wq1, sw1 = zq.zq_quantize_weight_groupwise(dev(w1), g, 8)
    wq2, sw2 = zq.zq_quantize_weight_groupwise(dev(w2), g, 8)
    xq, st, _ = zq.zq_layernorm_quant_tokenwise(dev(x), dev(gamma), dev(beta), 1e-5)
    h, acc1, _, _ = zq.zq_gemm_i8_dequant(xq, st, wq1, sw1, dev(b1), want_acc=True)
    hq, st2, y2 = zq.zq_gelu_quant_tokenwise(h, None, y_dtype=torch.float32)
    o, acc2, _, _ = zq.zq_gemm_i8_dequant(hq, st2, wq2, sw2, dev(b2), want_acc=True)
    torch.cuda.synchronize()
    a1 = orc.matmul_i32(host(xq), host(wq1))
    assert_bit_equal(host(acc1), a1, "acc1")
    ref1, mag1 = orc.dequant(a1, host(st), host(sw1), b1)
    assert_out_close(host(h), ref1, mag1, "h")
    q_o, s_o = orc.quant_tokenwise(host(y2))
    assert_bit_equal(host(hq), q_o, "hq")
    assert_bit_equal(host(st2), s_o, "st2")
    a2 = orc.matmul_i32(host(hq), host(wq2))
    assert_bit_equal(host(acc2), a2, "acc2")
    ref2, mag2 = orc.dequant(a2, host(st2), host(sw2), b2)
    assert_out_close(host(o), ref2, mag2, "o")
    # and the quantized layer tracks the fp64 layer it replaces
    y64, _ = orc.layernorm(x, gamma, beta, 1e-5)
    h64 = y64 @ w1.astype(np.float64).T + b1.astype(np.float64)
    g64 = 0.5 * h64 * (1 + np.vectorize(__import__("math").erf)(h64 / np.sqrt(2)))
    o64 = g64 @ w2.astype(np.float64).T + b2.astype(np.float64)
    rel = np.linalg.norm(host(o).astype(np.float64) - o64) / np.linalg.norm(o64)
    print("end-to-end relative error vs fp64 layer: %.4f" % rel, flush=True)
    assert rel < 0.05


# Full-size workloads, every (linear, token count) of the workload table: sampled rows against the
# oracle plus the Freivalds identity on every accumulator, in the launch configuration the benchmark times
# (default dispatch, a workspace of the size the library asks for).
FULL = [(name, M) for name in zq_inputs.LINEARS for M in zq_inputs.TOKENS[name.split("_")[0]]]
assert len(FULL) == 39


@pytest.mark.parametrize("name,M", FULL)
def test_full_size_workloads(zq, orc, name, M):
    K, N, g, bits = zq_inputs.LINEARS[name]
    nbytes = zq.gemm_workspace_bytes(M, N, K, bits)
    print("full", name, M, zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, bits, nbytes)), flush=True)
    _large_shape_check(zq, orc, name, M, N, K, g, bits, zq_inputs.rng_for(int(name[1]), M))


# The re-quantization of the output (token-wise codes of the FP16 tensor for the next GeMM) at full
# size: inside the tiled GeMM kernel at a prefill shape, by the second kernel behind the streaming
# schedule at a decode shape.  Every code and scale against the oracle's quantizer on the GPU's FP16 rows.
@pytest.mark.parametrize("name,M,in_kernel", [("c3_qkv", 2048, True), ("c5_qkv", 64, False), ("c2_ffc1", 4096, True)])
def test_full_size_requantization(zq, orc, name, M, in_kernel):
    K, N, g, bits = zq_inputs.LINEARS[name]
    print("full requant", name, M, flush=True)
    nbytes = zq.gemm_quant_workspace_bytes(M, N, K, bits)
    assert bool(zq.gemm_quantizes_in_kernel(M, N, K, bits, nbytes)) == in_kernel
    _large_shape_check(zq, orc, name, M, N, K, g, bits, zq_inputs.rng_for(int(name[1]), 9000 + M), requant=True)


# Token counts between decode and prefill on the workload matrices: the schedules with a K split
# (tiles above 64 tokens, streaming below) at sizes the oracle cannot cover element by element.
MID = [("c4_out", 192), ("c4_ffc2", 128), ("c4_ffc2", 320), ("c3_ffc2", 1024), ("c5_ffc2", 100), ("c3_out", 512)]


@pytest.mark.parametrize("name,M", MID)
def test_mid_token_counts_on_workload_matrices(zq, orc, name, M):
    K, N, g, bits = zq_inputs.LINEARS[name]
    nbytes = zq.gemm_workspace_bytes(M, N, K, bits)
    print("mid", name, M, zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, bits, nbytes)), flush=True)
    _large_shape_check(zq, orc, name, M, N, K, g, bits, zq_inputs.rng_for(int(name[1]), 7000 + M))


def _large_shape_check(zq, orc, name, M, N, K, g, bits, rng, requant=False):
    """Sampled rows against the oracle, the Freivalds identity on every accumulator, and the FP16
    output against the epilogue of the accumulators everywhere.  With requant also out_q / out_s_tok:
    every row against the oracle's token-wise quantizer applied to the FP16 output."""
    g_t = torch.Generator(device="cuda").manual_seed(zq_inputs.BASE_SEED + M)
    qmax = 127 if bits == 8 else 7
    xq_t = torch.randint(-127, 128, (M, K), generator=g_t, device="cuda", dtype=torch.int8)
    codes_t = torch.randint(-qmax, qmax + 1, (N, K), generator=g_t, device="cuda", dtype=torch.int8)
    if bits == 8:
        wq_t = codes_t
    else:
        u = codes_t.to(torch.uint8) & 0xF
        wq_t = (u[:, 0::2] | (u[:, 1::2] << 4)).contiguous()
    s_tok = zq_inputs.random_scales(rng, M, 5e-3, 0.3)
    s_w = zq_inputs.random_scales(rng, g, 1e-4, 1e-3)
    bias = zq_inputs.bias(rng, N, std=0.05)
    nbytes = zq.gemm_quant_workspace_bytes(M, N, K, bits) if requant else zq.gemm_workspace_bytes(M, N, K, bits)
    ws = zq.new_workspace(nbytes)
    fn = zq.zq_gemm_i8_dequant if bits == 8 else zq.zq_gemm_w4a8_dequant
    out, acc, out_q, out_s = fn(xq_t, dev(s_tok), wq_t, dev(s_w), dev(bias), want_acc=True, requant=requant,
                                workspace=ws)
    torch.cuda.synchronize()
    assert zq.quant_wait_expired(ws) == 0
    if requant:
        q_h, s_h, out_h = host(out_q), host(out_s), host(out)
        for m0 in range(0, M, 512):
            q_o, s_o = orc.quant_tokenwise(out_h[m0:m0 + 512].astype(np.float32))
            assert_bit_equal(s_h[m0:m0 + 512], s_o, name + " out_s_tok")
            assert_bit_equal(q_h[m0:m0 + 512], q_o, name + " out_q")
    freivalds_gpu(acc, xq_t, codes_t, seed=M + N)
    rows = np.unique(np.concatenate([[0, M - 1, M // 2], rng.integers(0, M, size=5),
                                     [min(M - 1, 255), min(M - 1, 256), min(M - 1, 127)]]))
    xq_h, codes_h = host(xq_t[torch.from_numpy(rows).cuda()]), host(codes_t)
    acc_o = orc.matmul_i32(xq_h, codes_h)
    acc_rows = host(acc[torch.from_numpy(rows).cuda()])
    assert_bit_equal(acc_rows, acc_o, name + " acc rows")
    ref, mag = orc.dequant(acc_o, s_tok[rows], s_w, bias)
    assert_out_close(host(out[torch.from_numpy(rows).cuda()]), ref, mag, name + " out rows")
    # the FP16 output must be the epilogue of the accumulator everywhere (library ops, fp64)
    gs = N // g
    step = max(1, (1 << 26) // N)
    sw_cols = torch.from_numpy(np.repeat(s_w.astype(np.float64), gs)).cuda()
    b64 = torch.from_numpy(bias.astype(np.float64)).cuda()
    st64 = torch.from_numpy(s_tok.astype(np.float64)).cuda()
    for m0 in range(0, M, step):
        p = acc[m0:m0 + step].to(torch.float64) * st64[m0:m0 + step, None] * sw_cols[None, :]
        err = (out[m0:m0 + step].to(torch.float64) - (p + b64[None, :])).abs()
        tol = 2e-3 * (p.abs() + b64.abs()[None, :]) + 2.0 ** -25
        assert bool((err <= tol).all()), name + " epilogue"


def test_autotune_registers_a_runnable_schedule(zq, orc):
    """The measured schedule table (App. D's offline ranking): whatever the tuner picks for a shape
    must reproduce the oracle's accumulators, and clearing the table restores the built-in choice."""
    from paper_2206_01861_amd import autotune
    rng = zq_inputs.rng_for(4, 79)
    for (M, N, K, g, bits) in [(16, 2048, 2048, 128, 8), (8, 1024, 4096, 64, 4)]:
        xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, bits)
        base = zq.gemm_choose_variant(M, N, K, bits, zq.gemm_workspace_bytes(M, N, K, bits))
        zq.tune_clear()
        try:
            entry, results = autotune.tune_shape(M, N, K, bits)
            assert len(results) >= 3 and entry["us"] == min(r["us"] for r in results)
            nbytes = zq.gemm_workspace_bytes(M, N, K, bits)
            assert zq.gemm_choose_variant(M, N, K, bits, nbytes) == entry["variant"]
            ws = zq.new_workspace(nbytes)
            res = _run(zq, bits, -1, xq, s_tok, wq, s_w, bias, workspace=ws)
            _check(orc, res, xq, s_tok, codes, s_w, bias, "tuned %dx%dx%d" % (M, N, K))
        finally:
            zq.tune_clear()
        assert zq.gemm_choose_variant(M, N, K, bits, zq.gemm_workspace_bytes(M, N, K, bits)) == base


def test_two_k_ranges_with_four_strips_per_workgroup(zq, orc):
    """The fullest workgroup of the two-range streaming schedule: four strips, eight consumer waves,
    strips dealt unevenly (65 over 17 row blocks).  The built-in cuts stop at three strips per
    workgroup where ranges apply, so the cut comes from the schedule table."""
    M, N, K, g = 8, 1040, 4096, 65
    rng = zq_inputs.rng_for(4, 83)
    xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, 8)
    zq.tune_clear()
    try:
        zq.tune_set(1, 32, N, K, 8, SKINNY, 17, 1)
        assert zq.gemm_stream_plan(M, N, K, 8, 0) == (17, 1, 4)
        assert zq.gemm_stream_k_ranges(M, N, K, 8, 0) == 2
        res = _run(zq, 8, -1, xq, s_tok, wq, s_w, bias)
        _check(orc, res, xq, s_tok, codes, s_w, bias, "two ranges, four strips")
    finally:
        zq.tune_clear()


def test_many_128_tiles_through_the_schedule_table(zq, orc):
    """128x128 tiles on a shape the built-in choice gives to larger tiles, reached the way a caller would:
    through an entry of the measured schedule table.  Twenty-one by twenty-one tiles, ragged everywhere."""
    M, N, K, g = 2600, 2576, 1024, 161
    rng = zq_inputs.rng_for(4, 91)
    for bits in (8, 4):
        xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, bits)
        zq.tune_clear()
        try:
            assert zq.gemm_choose_variant(M, N, K, bits, 0) != TILE128
            zq.tune_set(M, M, N, K, bits, TILE128)
            assert zq.gemm_choose_variant(M, N, K, bits, 0) == TILE128
            res = _run(zq, bits, -1, xq, s_tok, wq, s_w, bias)
            _check(orc, res, xq, s_tok, codes, s_w, bias, "tuned tile128 %d-bit" % bits)
        finally:
            zq.tune_clear()


def test_calls_on_two_streams_with_their_own_workspaces(zq, orc):
    """What the kernels of a call exchange lives in the caller's workspace, so calls on different
    workspaces may run at the same time: two K-split GeMMs and two GeMMs that quantize their output in
    the kernel, issued alternately on two streams several times over, must all give the oracle's bits."""
    rng = zq_inputs.rng_for(4, 92)
    split = []
    for (M, N, K, g) in [(32, 2048, 8192, 128), (16, 1040, 12288, 65)]:
        xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, 8)
        nbytes = zq.gemm_workspace_bytes(M, N, K, 8)
        assert zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, 8, nbytes)) == "skinny_splitk"
        split.append(dict(a=(dev(xq), dev(s_tok), dev(wq), dev(s_w), dev(bias)), ws=zq.new_workspace(nbytes),
                          h=(xq, s_tok, codes, s_w, bias), res=[]))
    quant = []
    for (M, N, K, g) in [(1024, 2048, 512, 64), (515, 1024, 1024, 64)]:
        xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, 8)
        ws = zq.new_workspace(zq.gemm_quant_workspace_bytes(M, N, K, 8))
        assert zq.gemm_quantizes_in_kernel(M, N, K, 8, ws.numel())
        quant.append(dict(a=(dev(xq), dev(s_tok), dev(wq), dev(s_w), dev(bias)), ws=ws,
                          h=(xq, s_tok, codes, s_w, bias), res=[]))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(6):
        for i in (0, 1):
            with torch.cuda.stream(streams[i]):
                split[i]["res"].append(zq.zq_gemm_i8_dequant(*split[i]["a"], want_acc=True, workspace=split[i]["ws"]))
                quant[i]["res"].append(zq.zq_gemm_i8_dequant(*quant[i]["a"], want_acc=True, requant=True,
                                                             workspace=quant[i]["ws"]))
    torch.cuda.synchronize()
    for c in split + quant:
        xq, s_tok, codes, s_w, bias = c["h"]
        acc_o = orc.matmul_i32(xq, codes)
        ref, mag = orc.dequant(acc_o, s_tok, s_w, bias)
        for rep, (out, acc, out_q, out_s) in enumerate(c["res"]):
            assert_bit_equal(host(acc), acc_o, "two streams acc rep %d" % rep)
            assert_out_close(host(out), ref, mag, "two streams out rep %d" % rep)
            if out_q is not None:
                q_o, s_o = orc.quant_tokenwise(host(out).astype(np.float32))
                assert_bit_equal(host(out_s), s_o, "two streams out_s_tok rep %d" % rep)
                assert_bit_equal(host(out_q), q_o, "two streams out_q rep %d" % rep)
        assert zq.quant_wait_expired(c["ws"]) == 0
