"""GeMM with bias + GeLU in its epilogue, then token-wise quantization (the fusion of Sec. 4.3's
bias-add + GeLU + quantization, moved into the dequantization epilogue of App. D), against the
oracle: the FP16 activation within tolerance of the fp64 chain, the codes and scales bit-exact
given that FP16 tensor."""
import numpy as np
import pytest
import torch

import zq_inputs
from helpers import assert_bit_equal, dev, host
from test_gpu_gemm import SIMPLE, SKINNY, SKINNY_SPLITK, TILE128, TILE256, TILE256X128, _case, orc, zq  # noqa: F401 (fixtures)

pytestmark = pytest.mark.gpu


def _check_fused(orc, g16, gq, s, xq, s_tok, codes, s_w, bias, approx, what):
    acc = orc.matmul_i32(xq, codes)
    ref, mag = orc.dequant(acc, s_tok, s_w, bias)             # fp64 pre-activation and its term magnitudes
    g_ref = orc.gelu_f64(ref, approx)
    # fp32 evaluation of the pre-activation (a few ulp of its terms), |GeLU'| <= 1.13, the
    # fp32 GeLU approximation (1.5e-7 absolute in Phi), then one FP16 rounding of the result.
    tol = 2e-3 * np.abs(g_ref) + 4e-6 * (mag + 1.0) + 2.0 ** -24
    err = np.abs(g16.astype(np.float64) - g_ref)
    assert (err <= tol).all(), "%s: g off by %.3e (tol %.3e), %d bad" % (
        what, err.max(), tol[np.unravel_index(err.argmax(), err.shape)], int((err > tol).sum()))
    q_o, s_o = orc.quant_tokenwise(g16.astype(np.float32))
    assert_bit_equal(s, s_o, what + " s_tok")
    assert_bit_equal(gq, q_o, what + " codes")


CASES = [
    (SIMPLE, 17, 768, 784, 48), (TILE128, 300, 400, 384, 25), (TILE128, 515, 1024, 1024, 64),
    (TILE256, 300, 528, 512, 33), (TILE256X128, 300, 400, 512, 25), (6, 300, 400, 512, 25), (SKINNY, 8, 6144, 2048, 128),
    (SKINNY, 100, 768, 768, 48), (SKINNY_SPLITK, 33, 2064, 8192, 3), (-1, 128, 4096, 1024, 64),
    (-1, 16, 4096, 1024, 64),
    # the tiled schedule with a K split: GeLU in the second kernel, then the row quantizer
    (7, 300, 400, 2048, 25), (-1, 192, 1024, 4096, 64),
]


@pytest.mark.parametrize("approx", [False, True])
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("variant,M,N,K,g", CASES)
def test_gemm_gelu_quant_against_oracle(zq, orc, variant, M, N, K, g, bits, approx):
    print("gemm+gelu", variant, bits, M, N, K, g, approx, flush=True)
    if bits == 4 and K % 32:
        pytest.skip("INT4 needs K % 32 == 0")
    rng = zq_inputs.rng_for(6, variant * 1000 + M + N + K + bits)
    xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, bits)
    # scales that put the pre-activation where GeLU bends: |u| of a few units
    s_tok = (s_tok * (3.0 / max(1e-9, float(np.sqrt(K)) * 40.0 * float(s_tok.mean()) * float(s_w.mean())))).astype(np.float32)
    nbytes = zq.gemm_workspace_bytes(M, N, K, bits)
    if variant in (SKINNY_SPLITK, 7) and nbytes == 0:
        pytest.skip("shape does not split")
    ws = zq.new_workspace(nbytes)
    if (variant, M) == (-1, 192):
        assert zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, bits, nbytes)) == "tile128_splitk"
        assert zq.gemm_quantizes_in_kernel(M, N, K, bits, nbytes) == 0
    prev = zq.force_gemm_variant(variant)
    try:
        g16, gq, s = zq.zq_gemm_gelu_quant_tokenwise(dev(xq), dev(s_tok), dev(wq), dev(s_w), dev(bias),
                                                     approx_tanh=approx, workspace=ws)
        torch.cuda.synchronize()
    finally:
        zq.force_gemm_variant(prev)
    assert zq.quant_wait_expired(ws) == 0
    _check_fused(orc, host(g16), host(gq), host(s), xq, s_tok, codes, s_w, bias, approx,
                 "fused %s %d-bit %dx%dx%d" % (zq.gemm_variant_name(variant), bits, M, N, K))


def test_fused_chain_tracks_two_call_chain(zq, orc):
    """The fused call and GeMM -> GeLU+quant differ only by the FP16 rounding of the pre-activation:
    codes agree except where that rounding moves a value across a quantization boundary."""
    rng = zq_inputs.rng_for(2, 9)
    M, H, F, g = 256, 1024, 4096, 64
    x = zq_inputs.config_activations("c2", rng, M, H)
    gamma, beta = zq_inputs.layernorm_params(rng, H)
    w1, b1 = zq_inputs.weights(rng, F, H), zq_inputs.bias(rng, F)
    wq1, sw1 = zq.zq_quantize_weight_groupwise(dev(w1), g, 8)
    xq, st, _ = zq.zq_layernorm_quant_tokenwise(dev(x), dev(gamma), dev(beta), 1e-5)
    h, _, _, _ = zq.zq_gemm_i8_dequant(xq, st, wq1, sw1, dev(b1))
    hq, st2, _ = zq.zq_gelu_quant_tokenwise(h, None)
    ws = zq.new_workspace(zq.gemm_quant_workspace_bytes(M, F, H, 8))
    g16, gq, s = zq.zq_gemm_gelu_quant_tokenwise(xq, st, wq1, sw1, dev(b1), workspace=ws)
    torch.cuda.synchronize()
    _check_fused(orc, host(g16), host(gq), host(s), host(xq), host(st), host(wq1), host(sw1), b1, False, "chain")
    rel_s = np.abs(host(s) - host(st2)) / host(st2)
    assert rel_s.max() < 2e-3
    diff = np.abs(host(gq).astype(np.int32) - host(hq).astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).mean() < 0.05


# (M, N, K, groups): both tile edges of the schedule that quantizes inside the GeMM kernel, ragged
# in M and N, bands of 2 to 40 tiles, one tile per band, K down to a single stage.
IN_KERNEL = [
    (300, 400, 384, 25), (129, 144, 64, 9), (515, 1024, 1024, 64), (1000, 2064, 256, 129),
    (2100, 5008, 128, 313), (4096, 4096, 1024, 64), (130, 8192, 128, 512), (5000, 272, 96, 17),
    (3000, 6160, 64, 385),      # more tiles than compute units: later bands start as earlier ones leave
]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,N,K,g", IN_KERNEL)
def test_in_kernel_quantization_equals_second_kernel(zq, orc, M, N, K, g, bits):
    """The GeMM kernel that quantizes its own output rows (row maxima exchanged between the tiles of
    a band) gives the bits of the two-kernel path: FP16 tensor, codes and scales; with and without
    the FP16 tensor; twice in a row (the exchange state must be back at zero); and for the plain
    GeMM's out_q.  Sampled rows are also checked against the oracle."""
    print("in-kernel quant", bits, M, N, K, g, flush=True)
    if bits == 4 and K % 32:
        pytest.skip("INT4 needs K % 32 == 0")
    rng = zq_inputs.rng_for(7, M + N + K + bits)
    xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, bits)
    s_tok = (s_tok * (3.0 / max(1e-9, float(np.sqrt(K)) * 40.0 * float(s_tok.mean()) * float(s_w.mean())))).astype(np.float32)
    args = (dev(xq), dev(s_tok), dev(wq), dev(s_w), dev(bias))
    gemm = zq.zq_gemm_i8_dequant if bits == 8 else zq.zq_gemm_w4a8_dequant
    ws = zq.new_workspace(0)                 # the fixed part is all the in-kernel quantization needs
    wsb = ws.numel()
    # small problems go to the untiled schedule by themselves: put them on a tiled one
    tiled = zq.gemm_choose_variant(M, N, K, bits, wsb) in (TILE128, TILE256)
    prev_variant = zq.force_gemm_variant(-1 if tiled else TILE128)
    try:
        assert zq.gemm_quantizes_in_kernel(M, N, K, bits, wsb)
        assert not zq.gemm_quantizes_in_kernel(M, N, K, bits, 0)         # no workspace: the second kernel
        if tiled:
            assert zq.gemm_quant_workspace_bytes(M, N, K, bits) == wsb
        g_ref, q_ref, s_ref = zq.zq_gemm_gelu_quant_tokenwise(*args)      # second-kernel path (no workspace)
        prev = zq.set_in_kernel_quant(False)
        try:
            assert not zq.gemm_quantizes_in_kernel(M, N, K, bits, wsb)
            o_ref, _, oq_ref, os_ref = gemm(*args, requant=True, workspace=ws)
            torch.cuda.synchronize()
        finally:
            zq.set_in_kernel_quant(prev)
        runs = []
        for rep in range(2):
            g1, q1, s1 = zq.zq_gemm_gelu_quant_tokenwise(*args, workspace=ws)
            g2, q2, s2 = zq.zq_gemm_gelu_quant_tokenwise(*args, keep_g=False, workspace=ws)
            o3, _, q3, s3 = gemm(*args, requant=True, workspace=ws)
            torch.cuda.synchronize()
            runs.append((g1, q1, s1, g2, q2, s2, o3, q3, s3))
    finally:
        zq.force_gemm_variant(prev_variant)
    for rep, (g1, q1, s1, g2, q2, s2, o3, q3, s3) in enumerate(runs):
        assert g2 is None
        assert_bit_equal(host(g1), host(g_ref), "g rep %d" % rep)
        assert_bit_equal(host(s1), host(s_ref), "s_tok rep %d" % rep)
        assert_bit_equal(host(q1), host(q_ref), "codes rep %d" % rep)
        assert_bit_equal(host(s2), host(s_ref), "s_tok without g rep %d" % rep)
        assert_bit_equal(host(q2), host(q_ref), "codes without g rep %d" % rep)
        assert_bit_equal(host(o3), host(o_ref), "plain GeMM out rep %d" % rep)
        assert_bit_equal(host(s3), host(os_ref), "plain GeMM out_s_tok rep %d" % rep)
        assert_bit_equal(host(q3), host(oq_ref), "plain GeMM out_q rep %d" % rep)
    assert zq.quant_wait_expired(ws) == 0
    rows = sorted(set([0, M - 1, M // 2, min(M - 1, 127), min(M - 1, 128), min(M - 1, 255), min(M - 1, 256)]))
    _check_fused(orc, host(g1)[rows], host(q1)[rows], host(s1)[rows], xq[rows], s_tok[rows], codes, s_w, bias, False,
                 "in-kernel %d-bit %dx%dx%d" % (bits, M, N, K))


def test_missing_fp16_output_needs_the_in_kernel_path(zq):
    """Without a buffer for g the call is only legal where the GeMM kernel quantizes; elsewhere it
    is refused before anything is launched."""
    M, N, K, g = 8, 256, 256, 16
    assert not zq.gemm_quantizes_in_kernel(M, N, K, 8)
    xq = torch.zeros((M, K), dtype=torch.int8, device="cuda")
    wq = torch.zeros((N, K), dtype=torch.int8, device="cuda")
    st = torch.ones(M, device="cuda")
    sw = torch.ones(g, device="cuda")
    with pytest.raises(zq.ZQError) as e:
        zq.zq_gemm_gelu_quant_tokenwise(xq, st, wq, sw, keep_g=False)
    assert e.value.code == 4


def test_in_kernel_quantization_under_graph_replay(zq, orc):
    """The launch generation of the in-kernel quantizer lives on the device, so a captured call can
    be replayed: every replay, with new inputs copied into the captured buffers and eager calls of
    other shapes in between, must give the bits of the two-kernel path on the same inputs."""
    M, N, K, g = 1024, 2048, 512, 64
    ws = zq.new_workspace(0)
    ws2 = zq.new_workspace(0)                # the eager calls between the replays use their own
    assert zq.gemm_quantizes_in_kernel(M, N, K, 8, ws.numel())
    rng = zq_inputs.rng_for(8, 1)
    _, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, 8)
    s_tok = (s_tok * (3.0 / max(1e-9, float(np.sqrt(K)) * 40.0 * float(s_tok.mean()) * float(s_w.mean())))).astype(np.float32)
    xq_d = torch.zeros((M, K), dtype=torch.int8, device="cuda")
    st_d, wq_d, sw_d, b_d = dev(s_tok), dev(wq), dev(s_w), dev(bias)
    gq = torch.empty((M, N), dtype=torch.int8, device="cuda")
    s2 = torch.empty(M, dtype=torch.float32, device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        zq.zq_gemm_gelu_quant_tokenwise(xq_d, st_d, wq_d, sw_d, b_d, out=(None, gq, s2), keep_g=False, workspace=ws)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            zq.zq_gemm_gelu_quant_tokenwise(xq_d, st_d, wq_d, sw_d, b_d, out=(None, gq, s2), keep_g=False,
                                            workspace=ws)
    torch.cuda.synchronize()
    other = _case(zq_inputs.rng_for(8, 2), 300, 400, 384, 25, 8)
    for rep in range(4):
        xq = zq_inputs.random_codes(zq_inputs.rng_for(8, 10 + rep), (M, K))
        xq_d.copy_(dev(xq))
        gq.zero_()
        s2.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_q, got_s = host(gq).copy(), host(s2).copy()
        # eager work of another shape between the replays, on the in-kernel path as well
        prev_v = zq.force_gemm_variant(TILE128)
        try:
            zq.zq_gemm_gelu_quant_tokenwise(dev(other[0]), dev(other[1]), dev(other[5]), dev(other[2]), dev(other[3]),
                                            workspace=ws2 if rep % 2 else ws)
        finally:
            zq.force_gemm_variant(prev_v)
        g_ref, q_ref, s_ref = zq.zq_gemm_gelu_quant_tokenwise(xq_d, st_d, wq_d, sw_d, b_d)   # second-kernel path
        torch.cuda.synchronize()
        assert_bit_equal(got_s, host(s_ref), "replay %d s_tok" % rep)
        assert_bit_equal(got_q, host(q_ref), "replay %d codes" % rep)
        if rep == 0:                         # and the replayed bits are the oracle's, given the FP16 tensor
            _check_fused(orc, host(g_ref)[:64], got_q[:64], got_s[:64], xq[:64], s_tok[:64], codes, s_w, bias, False,
                         "replayed in-kernel quantization")
    assert zq.quant_wait_expired(ws) == 0 and zq.quant_wait_expired(ws2) == 0


def test_in_kernel_quantization_while_another_stream_keeps_the_chip_busy(zq, orc):
    """Tiles wait for the other tiles of their band, which is only safe because workgroups start in
    id order: with another stream's GeMMs taking compute units away at the same time the call must
    still finish with the right bits and without any wait running out."""
    M, N, K, g = 4096, 4096, 512, 64
    rng = zq_inputs.rng_for(9, 1)
    xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, 8)
    s_tok = (s_tok * (3.0 / max(1e-9, float(np.sqrt(K)) * 40.0 * float(s_tok.mean()) * float(s_w.mean())))).astype(np.float32)
    args = (dev(xq), dev(s_tok), dev(wq), dev(s_w), dev(bias))
    ws = zq.new_workspace(0)
    assert zq.gemm_quantizes_in_kernel(M, N, K, 8, ws.numel())
    _, q_ref, s_ref = zq.zq_gemm_gelu_quant_tokenwise(*args)             # second-kernel path
    torch.cuda.synchronize()
    a = torch.randn((4096, 4096), device="cuda", dtype=torch.float16)
    side = torch.cuda.Stream()
    outs = []
    with torch.cuda.stream(side):
        for _ in range(40):
            b = a @ a                                   # ~0.1 ms each on the other stream
    for _ in range(12):
        outs.append(zq.zq_gemm_gelu_quant_tokenwise(*args, keep_g=False, workspace=ws))
    torch.cuda.synchronize()
    assert zq.quant_wait_expired(ws) == 0
    for i, (_, q, s) in enumerate(outs):
        assert_bit_equal(host(s), host(s_ref), "call %d s_tok" % i)
        assert_bit_equal(host(q), host(q_ref), "call %d codes" % i)
