"""HIP-graph replay of the quantized linear layer (App. D replays a captured graph for small-model
inference): the chains of workload c1 (LayerNorm+quant -> GeMM 768 -> 768 at 128 tokens) and c2
(LayerNorm+quant -> GeMM -> GeLU+quant -> GeMM on the BERT-large feed-forward pair at 4096 tokens)
are captured once and replayed with new inputs; after every replay each stage is checked against
the oracle, fed with the previous stage's GPU result, exactly as the eager tests do.  Eager calls
on the same library run between the replays."""
import numpy as np
import pytest
import torch

import zq_inputs
from helpers import assert_bit_equal, assert_out_close, check_fused_codes, dev, host
from test_gpu_gemm import orc, zq  # noqa: F401 (fixtures)
from test_gpu_gemm_gelu import _check_fused

pytestmark = pytest.mark.gpu


def _capture(fn):
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        fn()                                      # warm up outside the capture (kernel attributes are set here)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            fn()
    torch.cuda.synchronize()
    return graph


def _eager_noise(zq):
    """Unrelated eager work between replays: a K-split GeMM and a front-end call of other shapes."""
    rng = zq_inputs.rng_for(3, 1)
    xq = dev(zq_inputs.random_codes(rng, (8, 8192)))
    wq = dev(zq_inputs.random_codes(rng, (512, 8192)))
    ws = zq.new_workspace(zq.gemm_workspace_bytes(8, 512, 8192, 8))
    zq.zq_gemm_i8_dequant(xq, torch.ones(8, device="cuda"), wq, torch.ones(32, device="cuda"), workspace=ws)
    zq.zq_quantize_tokenwise(torch.randn((33, 1024), device="cuda").half())
    torch.cuda.synchronize()


def test_c1_chain_under_graph_replay(zq, orc):
    M, H, g = 128, 768, 48
    rng = zq_inputs.rng_for(1, 3)
    gamma, beta = zq_inputs.layernorm_params(rng, H)
    w, b = zq_inputs.weights(rng, H, H), zq_inputs.bias(rng, H)
    wq, sw = zq.zq_quantize_weight_groupwise(dev(w), g, 8)
    wq_o, sw_o, _ = orc.quantize_weight_groupwise(w, g, 8)
    assert_bit_equal(host(wq), wq_o, "wq")
    assert_bit_equal(host(sw), sw_o, "s_w")
    x_d = torch.zeros((M, H), dtype=torch.float16, device="cuda")
    gamma_d, beta_d, b_d = dev(gamma), dev(beta), dev(b)
    xq = torch.empty((M, H), dtype=torch.int8, device="cuda")
    st = torch.empty(M, dtype=torch.float32, device="cuda")
    out = torch.empty((M, H), dtype=torch.float16, device="cuda")
    acc = torch.empty((M, H), dtype=torch.int32, device="cuda")
    taps = {}

    def chain():
        _, _, taps["y"] = zq.zq_layernorm_quant_tokenwise(x_d, gamma_d, beta_d, 1e-5, y_dtype=torch.float32,
                                                          out=(xq, st))
        zq.zq_gemm_i8_dequant(xq, st, wq, sw, b_d, out=out, acc_out=acc)

    graph = _capture(chain)
    for rep in range(3):
        x = zq_inputs.config_activations("c1", zq_inputs.rng_for(1, 10 + rep), M, H)
        x_d.copy_(dev(x))
        for t in (xq, st, out, acc):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        what = "c1 replay %d " % rep
        y64, _ = orc.layernorm(x, gamma, beta, 1e-5)
        check_fused_codes(host(xq), host(st), host(taps["y"]), y64, what + "LayerNorm")
        q_o, s_o = orc.quant_tokenwise(host(taps["y"]))
        assert_bit_equal(host(xq), q_o, what + "xq")
        assert_bit_equal(host(st), s_o, what + "s_tok")
        acc_o = orc.matmul_i32(host(xq), wq_o)
        assert_bit_equal(host(acc), acc_o, what + "acc")
        ref, mag = orc.dequant(acc_o, host(st), sw_o, b)
        assert_out_close(host(out), ref, mag, what + "out")
        _eager_noise(zq)


def test_c2_chain_under_graph_replay(zq, orc):
    M, H, F, g = 4096, 1024, 4096, 64
    rng = zq_inputs.rng_for(2, 3)
    gamma, beta = zq_inputs.layernorm_params(rng, H)
    w1, b1 = zq_inputs.weights(rng, F, H), zq_inputs.bias(rng, F)
    w2, b2 = zq_inputs.weights(rng, H, F), zq_inputs.bias(rng, H)
    wq1, sw1 = zq.zq_quantize_weight_groupwise(dev(w1), g, 8)
    wq2, sw2 = zq.zq_quantize_weight_groupwise(dev(w2), g, 8)
    wq1_h, sw1_h, wq2_h, sw2_h = host(wq1), host(sw1), host(wq2), host(sw2)
    assert_bit_equal(wq1_h, orc.quantize_weight_groupwise(w1, g, 8)[0], "wq1")
    assert_bit_equal(wq2_h, orc.quantize_weight_groupwise(w2, g, 8)[0], "wq2")
    x_d = torch.zeros((M, H), dtype=torch.float16, device="cuda")
    gamma_d, beta_d, b1_d, b2_d = dev(gamma), dev(beta), dev(b1), dev(b2)
    xq = torch.empty((M, H), dtype=torch.int8, device="cuda")
    st = torch.empty(M, dtype=torch.float32, device="cuda")
    h = torch.empty((M, F), dtype=torch.float16, device="cuda")
    acc1 = torch.empty((M, F), dtype=torch.int32, device="cuda")
    hq = torch.empty((M, F), dtype=torch.int8, device="cuda")
    st2 = torch.empty(M, dtype=torch.float32, device="cuda")
    o = torch.empty((M, H), dtype=torch.float16, device="cuda")
    acc2 = torch.empty((M, H), dtype=torch.int32, device="cuda")
    # the three-call chain of the same layer (GeLU and the quantizer inside the first GeMM kernel)
    ws = zq.new_workspace(zq.gemm_quant_workspace_bytes(M, F, H, 8))
    assert zq.gemm_quantizes_in_kernel(M, F, H, 8, ws.numel())
    g16 = torch.empty((M, F), dtype=torch.float16, device="cuda")
    gq = torch.empty((M, F), dtype=torch.int8, device="cuda")
    gs = torch.empty(M, dtype=torch.float32, device="cuda")
    o3 = torch.empty((M, H), dtype=torch.float16, device="cuda")
    acc3 = torch.empty((M, H), dtype=torch.int32, device="cuda")
    taps = {}

    def chain():
        _, _, taps["y"] = zq.zq_layernorm_quant_tokenwise(x_d, gamma_d, beta_d, 1e-5, y_dtype=torch.float32,
                                                          out=(xq, st))
        zq.zq_gemm_i8_dequant(xq, st, wq1, sw1, b1_d, out=h, acc_out=acc1)
        _, _, taps["y2"] = zq.zq_gelu_quant_tokenwise(h, None, y_dtype=torch.float32, out=(hq, st2))
        zq.zq_gemm_i8_dequant(hq, st2, wq2, sw2, b2_d, out=o, acc_out=acc2)
        zq.zq_gemm_gelu_quant_tokenwise(xq, st, wq1, sw1, b1_d, workspace=ws, out=(g16, gq, gs))
        zq.zq_gemm_i8_dequant(gq, gs, wq2, sw2, b2_d, out=o3, acc_out=acc3)

    graph = _capture(chain)
    rows = np.array([0, 1, 127, 128, 255, 256, 2047, 4095])       # stage checks that need fp64 work on the host
    for rep in range(2):
        x = zq_inputs.config_activations("c2", zq_inputs.rng_for(2, 10 + rep), M, H)
        x_d.copy_(dev(x))
        for t in (xq, st, h, acc1, hq, st2, o, acc2, g16, gq, gs, o3, acc3):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        what = "c2 replay %d " % rep
        y64, _ = orc.layernorm(x[rows], gamma, beta, 1e-5)
        check_fused_codes(host(xq)[rows], host(st)[rows], host(taps["y"])[rows], y64, what + "LayerNorm")
        q_o, s_o = orc.quant_tokenwise(host(taps["y"]))
        assert_bit_equal(host(xq), q_o, what + "xq")
        assert_bit_equal(host(st), s_o, what + "s_tok")
        a1 = orc.matmul_i32(host(xq), wq1_h)
        assert_bit_equal(host(acc1), a1, what + "acc1")
        ref1, mag1 = orc.dequant(a1, host(st), sw1_h, b1)
        assert_out_close(host(h), ref1, mag1, what + "h")
        g64, _ = orc.gelu(host(h)[rows], None)
        check_fused_codes(host(hq)[rows], host(st2)[rows], host(taps["y2"])[rows], g64, what + "GeLU")
        q_o, s_o = orc.quant_tokenwise(host(taps["y2"]))
        assert_bit_equal(host(hq), q_o, what + "hq")
        assert_bit_equal(host(st2), s_o, what + "s_tok2")
        a2 = orc.matmul_i32(host(hq), wq2_h)
        assert_bit_equal(host(acc2), a2, what + "acc2")
        ref2, mag2 = orc.dequant(a2, host(st2), sw2_h, b2)
        assert_out_close(host(o), ref2, mag2, what + "o")
        # three-call chain: the activated tensor against gelu(dequant(acc1)) in fp64, its codes given that tensor
        _check_fused(orc, host(g16)[rows], host(gq)[rows], host(gs)[rows], host(xq)[rows], host(st)[rows], wq1_h, sw1_h,
                     b1, False, what + "fused GeMM 1")
        q_o, s_o = orc.quant_tokenwise(host(g16).astype(np.float32))
        assert_bit_equal(host(gq), q_o, what + "gq")
        assert_bit_equal(host(gs), s_o, what + "gs")
        a3 = orc.matmul_i32(host(gq), wq2_h)
        assert_bit_equal(host(acc3), a3, what + "acc3")
        ref3, mag3 = orc.dequant(a3, host(gs), sw2_h, b2)
        assert_out_close(host(o3), ref3, mag3, what + "o3")
        assert zq.quant_wait_expired(ws) == 0
        _eager_noise(zq)
