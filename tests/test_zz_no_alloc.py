"""The entry point that allocates nothing (zq_gemm_i8_dequant_static: the library's static scratch
buffer stands in for the caller's workspace) against zq_gemm_i8_dequant on the same inputs: INT32
accumulators, FP16 output, codes and scales bit for bit, and against the oracle.  Two calls in a
row, the second with a smaller input, for the two kinds of schedule that use the scratch (a K split
across workgroups, and the tiled kernel that quantizes its own output)."""
import numpy as np
import pytest
import torch

import zq_inputs
from helpers import assert_bit_equal, assert_out_close, dev, host
from test_gpu_gemm import _case, orc, zq  # noqa: F401 (fixtures)

pytestmark = pytest.mark.gpu


def _pair(zq, orc, M, N, K, g, requant, seed):
    rng = zq_inputs.rng_for(5, seed)
    xq, s_tok, s_w, bias, codes, wq = _case(rng, M, N, K, g, 8)
    args = (dev(xq), dev(s_tok), dev(wq), dev(s_w), dev(bias))
    need = zq.gemm_quant_workspace_bytes(M, N, K, 8) if requant else zq.gemm_workspace_bytes(M, N, K, 8)
    assert zq.WORKSPACE_FIXED_BYTES <= need <= zq.STATIC_SCRATCH_BYTES, "the case must use the scratch"
    ws = zq.new_workspace(need)
    o_ref, a_ref, q_ref, s_ref = zq.zq_gemm_i8_dequant(*args, want_acc=True, requant=requant, workspace=ws)
    # every output buffer is the caller's: the call under test allocates nothing
    out = torch.empty((M, N), dtype=torch.float16, device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    oq = torch.empty((M, N), dtype=torch.int8, device="cuda") if requant else None
    os_ = torch.empty(M, dtype=torch.float32, device="cuda") if requant else None
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    zq.zq_gemm_i8_dequant_static(*args, out=out, acc_out=acc, out_q=oq, out_s_tok=os_)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    what = "static %dx%dx%d" % (M, N, K)
    assert_bit_equal(host(acc), host(a_ref), what + " acc")
    assert_bit_equal(host(out), host(o_ref), what + " out")
    acc_o = orc.matmul_i32(xq, codes)
    assert_bit_equal(host(acc), acc_o, what + " acc vs oracle")
    ref, mag = orc.dequant(acc_o, s_tok, s_w, bias)
    assert_out_close(host(out), ref, mag, what + " out vs oracle")
    if requant:
        assert_bit_equal(host(os_), host(s_ref), what + " out_s_tok")
        assert_bit_equal(host(oq), host(q_ref), what + " out_q")
        q_o, s_o = orc.quant_tokenwise(host(out).astype(np.float32))
        assert_bit_equal(host(os_), s_o, what + " out_s_tok vs oracle")
        assert_bit_equal(host(oq), q_o, what + " out_q vs oracle")


def test_static_scratch_k_split_then_a_smaller_one(zq, orc):
    for i, (M, N, K, g) in enumerate([(32, 2048, 8192, 128), (8, 512, 8192, 32)]):
        print("static scratch, K split", M, N, K, flush=True)
        assert zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, 8, zq.STATIC_SCRATCH_BYTES)) == "skinny_splitk"
        _pair(zq, orc, M, N, K, g, False, 10 + i)


def test_static_scratch_in_kernel_quantization_then_a_smaller_one(zq, orc):
    for i, (M, N, K, g) in enumerate([(1024, 2048, 512, 64), (515, 1024, 256, 64)]):
        print("static scratch, in-kernel quantization", M, N, K, flush=True)
        assert zq.gemm_quantizes_in_kernel(M, N, K, 8, zq.STATIC_SCRATCH_BYTES)
        _pair(zq, orc, M, N, K, g, True, 20 + i)


def test_static_scratch_refuses_what_it_cannot_hold(zq):
    M, N, K = 1024, 2048, 8192
    assert zq.gemm_workspace_bytes(M, N, K, 8) > zq.STATIC_SCRATCH_BYTES
    xq = torch.zeros((M, K), dtype=torch.int8, device="cuda")
    wq = torch.zeros((N, K), dtype=torch.int8, device="cuda")
    with pytest.raises(zq.ZQError) as e:
        zq.zq_gemm_i8_dequant_static(xq, torch.ones(M, device="cuda"), wq, torch.ones(128, device="cuda"))
    assert e.value.code == 6
