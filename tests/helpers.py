"""Shared test utilities: host<->device moves and the comparison rules of the
parity contract.  No method arithmetic lives here; expected values always come
from oracle/."""
import numpy as np
import torch


def dev(a):
    """numpy array -> CUDA tensor (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def assert_bit_equal(got, want, what):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if got.dtype.kind == "f":
        same = got.view(np.uint32 if got.dtype == np.float32 else np.uint16) == \
            want.view(np.uint32 if want.dtype == np.float32 else np.uint16)
    else:
        same = got == want
    if not same.all():
        bad = np.argwhere(~same)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d differ; first at %s: got %r want %r"
                             % (what, len(bad), same.size, i, got[i], want[i]))


def assert_out_close(out16, ref64, mag64, what, rel=2e-3):
    """FP16 output against the fp64 reference: |out - ref| <= rel * (|acc*s*s| + |bias|),
    plus half an fp16 subnormal step for values that underflow."""
    out = np.asarray(out16).astype(np.float64)
    err = np.abs(out - ref64)
    tol = rel * mag64 + 2.0 ** -25
    if not (err <= tol).all():
        i = tuple(np.argwhere(err > tol)[0])
        raise AssertionError("%s: out %r ref %r err %.3e tol %.3e at %s (%d bad)"
                             % (what, out[i], ref64[i], err[i], tol[i], i, int((err > tol).sum())))


def check_fused_codes(xq_gpu, s_gpu, y_gpu32, y64, what):
    """Tier-2 rule for codes produced behind a fused fp32 operator, against the fp64 chain.

    y: |y_gpu - y64| <= 1e-5 * (|y64| + rms_row).
    scale: relative difference <= 1e-5.
    codes: every mismatch is one step and sits within 2e-3 of a rounding tie of the fp64 value.
    Returns the number of mismatching codes."""
    from oracle import zq_oracle as orc
    rms = np.sqrt((y64 ** 2).mean(axis=1, keepdims=True))
    if y_gpu32 is not None:
        bad = np.abs(y_gpu32.astype(np.float64) - y64) > 1e-5 * (np.abs(y64) + rms) + 1e-30
        assert not bad.any(), "%s: y differs at %d places" % (what, int(bad.sum()))
    xq_o, s_o = orc.quant_tokenwise(y64.astype(np.float32))
    denom = np.maximum(np.abs(s_o), 1e-30)
    assert (np.abs(s_gpu - s_o) / denom <= 1e-5).all(), what + ": s_tok"
    diff = xq_gpu.astype(np.int32) - xq_o.astype(np.int32)
    mism = diff != 0
    if mism.any():
        assert np.abs(diff).max() == 1, what + ": a code is off by more than one step"
        a = np.abs(y64).max(axis=1, keepdims=True)
        t = y64 * (127.0 / np.maximum(a, 1e-300))
        frac = np.abs(t - (np.floor(t) + 0.5))
        assert (frac[mism] <= 2e-3).all(), what + ": a mismatch is not at a rounding tie"
    return int(mism.sum())


def freivalds_gpu(acc_t, xq_t, wq_codes_t, seed, trials=2):
    """Exact check of acc == xq @ wq^T without forming the product:
    sum_n acc[m,n] r[n] == sum_k xq[m,k] (sum_n wq[n,k] r[n]) in int64, random r.
    All sums use torch's elementwise int64 ops (library code, not ours)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    N = acc_t.shape[1]
    for _ in range(trials):
        r = torch.randint(-2 ** 15, 2 ** 15, (N,), generator=g, dtype=torch.int64).cuda()
        lhs = torch.zeros(acc_t.shape[0], dtype=torch.int64, device="cuda")
        step = max(1, (1 << 27) // N)
        for m0 in range(0, acc_t.shape[0], step):
            lhs[m0:m0 + step] = (acc_t[m0:m0 + step].to(torch.int64) * r[None, :]).sum(dim=1)
        K = wq_codes_t.shape[1]
        v = torch.zeros(K, dtype=torch.int64, device="cuda")
        stepn = max(1, (1 << 27) // K)
        for n0 in range(0, N, stepn):
            v += (wq_codes_t[n0:n0 + stepn].to(torch.int64) * r[n0:n0 + stepn, None]).sum(dim=0)
        rhs = torch.zeros_like(lhs)
        stepm = max(1, (1 << 27) // K)
        for m0 in range(0, xq_t.shape[0], stepm):
            rhs[m0:m0 + stepm] = (xq_t[m0:m0 + stepm].to(torch.int64) * v[None, :]).sum(dim=1)
        if not torch.equal(lhs, rhs):
            bad = torch.nonzero(lhs != rhs).flatten()
            raise AssertionError("Freivalds identity fails on %d rows, first %d" % (bad.numel(), int(bad[0])))
