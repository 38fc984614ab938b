"""The measurement probes of include/zq_probe.h on the GPU: they are not steps of the quantized layer, so
there is no oracle value to match; what is checked is that every probe runs to completion inside its
buffers and that the results that are defined have their defined value (the matrix-core probe computes
real products: against the oracle's integer GeMM on one thread's operands)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zq():
    import paper_2206_01861_amd as lib
    lib.lib()
    return lib


def test_read_stream_leaves_the_sink_alone(zq):
    buf = torch.randint(0, 256, (8 << 20,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    zq.zq_probe_read_stream(buf, sink)
    zq.zq_probe_read_stream(buf[:4096], sink)
    torch.cuda.synchronize()
    assert int(sink.to(torch.int32).sum()) == 0        # written only if the data sum to a magic value


def test_mfma_probe_sums_real_products(zq):
    """Every wave multiplies its own four by four operand fragments `iters` times over; the sink holds, per
    thread, the sum of its accumulator registers folded four ways.  Summed over a wave that is the sum of all
    entries of the 128 x 128 product of the wave's operands, times iters: checked with numpy on int64."""
    blocks, iters = 4, 3
    ops = torch.randint(-127, 128, (blocks * 256 * 128,), dtype=torch.int8, device="cuda")
    sink = torch.zeros(blocks * 256 * 16, dtype=torch.uint8, device="cuda")
    n = zq.zq_probe_mfma_i8(ops.view(torch.uint8), blocks, iters, sink)
    torch.cuda.synchronize()
    assert n == blocks * 4 * iters * 16 * 65536
    got = sink.view(torch.int32).to(torch.int64).view(blocks * 4, 64 * 4).sum(dim=1).cpu().numpy()
    o = ops.cpu().numpy().astype(np.int64).reshape(blocks * 4, 64, 8, 16)      # wave, lane, fragment, byte
    # lane l supplies row l % 32 and the 16-byte half l // 32 of the 32-byte k step of every fragment
    a = o[:, :, :4, :].reshape(blocks * 4, 2, 32, 4, 16).transpose(0, 3, 2, 1, 4).reshape(blocks * 4, 128, 32)
    b = o[:, :, 4:, :].reshape(blocks * 4, 2, 32, 4, 16).transpose(0, 3, 2, 1, 4).reshape(blocks * 4, 128, 32)
    want = np.array([(a[w] @ b[w].T).sum() for w in range(blocks * 4)]) * iters
    assert (got == want).all()
    # zero operands: zero sums
    zq.zq_probe_mfma_i8(torch.zeros_like(ops).view(torch.uint8), blocks, iters, sink)
    torch.cuda.synchronize()
    assert int(sink.view(torch.int32).abs().sum()) == 0


def test_tile_traffic_probe_runs_inside_its_buffers(zq):
    """The waves of this probe are not ordered against the loads that refill their LDS, so only the all-zero
    case has a defined result; canaries around the source and the sink show that nothing else is written."""
    blocks, iters = 8, 5
    pad = 4096
    src_all = torch.zeros((2 << 20) + 2 * pad, dtype=torch.uint8, device="cuda")
    sink_all = torch.full((blocks * 512 * 16 + 2 * pad,), 0x5a, dtype=torch.uint8, device="cuda")
    src, sink = src_all[pad:pad + (2 << 20)], sink_all[pad:pad + blocks * 512 * 16]
    n = zq.zq_probe_mfma_i8_tile_traffic(src, blocks, iters, sink)
    torch.cuda.synchronize()
    assert n == blocks * 8 * iters * 32 * 65536
    assert int(sink.to(torch.int32).sum()) == 0
    assert bool((sink_all[:pad] == 0x5a).all()) and bool((sink_all[-pad:] == 0x5a).all())
    src.random_(0, 256)
    before = src_all.clone()
    zq.zq_probe_mfma_i8_tile_traffic(src, blocks, iters, sink)
    torch.cuda.synchronize()
    assert torch.equal(src_all, before)
    assert bool((sink_all[:pad] == 0x5a).all()) and bool((sink_all[-pad:] == 0x5a).all())
