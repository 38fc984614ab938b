"""Pins for the oracle's quantizer (App. A.2; Sec. 4.1 group-wise / token-wise).

The paper prints no worked numeric example, so the quantizer is pinned by what
the definition and the mathematics fix: hand-derived cases, exact-rational brute
force over every fp16 value, invariants, symmetries and the group geometry.
None of these retype the oracle's formula in fp32; the references are exact
rational arithmetic or closed forms.
"""
from fractions import Fraction

import numpy as np
import pytest

import zq_inputs
from oracle import zq_oracle as orc


def _rne_fraction(t):
    """Round an exact rational half-to-even."""
    fl = t.numerator // t.denominator
    r = t - fl
    if r > Fraction(1, 2):
        return fl + 1
    if r < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def test_half_to_float_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    got = orc.half_to_float(h)
    want = h.astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


@pytest.mark.parametrize("qmax,want,scale", [
    # absmax = 1 -> inv = qmax exactly, products exact: 127, -63.5, 31.75, 12.7
    (127, [127, -64, 32, 13], Fraction(1, 127)),
    # 7, -3.5, 1.75, 0.7
    (7, [7, -4, 2, 1], Fraction(1, 7)),
])
def test_hand_worked_example(qmax, want, scale):
    q, s = orc.quantize_block(np.array([1.0, -0.5, 0.25, 0.1], np.float32), qmax)
    assert q.tolist() == want
    # fp32 nearest to the exact scale
    assert abs(Fraction(float(s)) - scale) <= Fraction(1, 2 ** 24) * scale


def test_ties_go_to_even_when_scale_is_one():
    # absmax = qmax makes inv = 1 exactly, so codes are RNE of the inputs themselves.
    v = np.array([127.0, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 62.5, 63.5, -126.5, 0.49, 0.51],
                 np.float32)
    q, s = orc.quantize_block(v, 127)
    assert q.tolist() == [127, 0, 2, 2, 4, 0, -2, -2, 62, 64, -126, 0, 1]
    assert s == np.float32(1.0)
    v4 = np.array([7.0, 0.5, 1.5, 2.5, -3.5, -6.5, 6.5], np.float32)
    q4, s4 = orc.quantize_block(v4, 7)
    assert q4.tolist() == [7, 0, 2, 2, -4, -6, 6]
    assert s4 == np.float32(1.0)


@pytest.mark.parametrize("qmax", [127, 7])
@pytest.mark.parametrize("absmax", [1.0, 0.02, 3.1416, 35.0, 6.1e-5, 60000.0])
def test_every_fp16_value_against_exact_rational(qmax, absmax):
    """All finite fp16 v with |v| <= a: the code is RNE(v*qmax/a) computed exactly,
    except within the fp32 rounding band of a tie, where either neighbour is allowed."""
    a = np.float16(absmax)
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    keep = np.isfinite(h) & (np.abs(h.astype(np.float32)) <= np.float32(a))
    v = np.concatenate([[a], h[keep]]).astype(np.float16)
    v32 = v.astype(np.float32)
    q, s = orc.quantize_block(v32, qmax)
    fa = Fraction(float(a))
    assert abs(Fraction(float(s)) - fa / qmax) <= (fa / qmax) * Fraction(1, 2 ** 24)
    band = Fraction(qmax, 2 ** 22)      # two fp32 roundings of a value <= qmax
    n_tie = 0
    for vi, qi in zip(v32.tolist(), q.tolist()):
        t = Fraction(vi) * qmax / fa
        want = _rne_fraction(t)
        if qi != want:
            assert abs(t - qi) <= Fraction(1, 2) + band, (vi, qi, float(t))
            n_tie += 1
        assert -qmax <= qi <= qmax
    assert q[0] == qmax
    assert n_tie <= 8


@pytest.mark.parametrize("qmax", [127, 7])
def test_invariants_on_workload_shaped_rows(qmax):
    rng = zq_inputs.rng_for(9, 1)
    x = zq_inputs.activations(rng, 64, 768, n_outliers=4, outlier_scale=20.0,
                              token_spread=True).astype(np.float32)
    for row in x:
        q, s = orc.quantize_block(row, qmax)
        a = np.abs(row).max()
        # reconstruction error at most half a step (plus the fp32 slack of inv)
        err = np.abs(row.astype(np.float64) - float(s) * q.astype(np.float64))
        assert err.max() <= float(s) / 2 * (1 + 1e-4)
        # the extreme element maps to +-qmax, nothing leaves the symmetric range
        i = int(np.argmax(np.abs(row)))
        assert q[i] == (qmax if row[i] > 0 else -qmax)
        assert q.min() >= -qmax and q.max() <= qmax
        assert abs(float(s) * qmax - float(a)) <= float(a) * 2.0 ** -23
        # monotone: larger input never gets a smaller code
        order = np.argsort(row, kind="stable")
        assert np.all(np.diff(q[order].astype(np.int32)) >= 0)


def test_power_of_two_scaling_and_odd_symmetry_and_idempotence():
    rng = zq_inputs.rng_for(9, 2)
    v = rng.standard_normal(4096).astype(np.float16).astype(np.float32)
    q, s = orc.quantize_block(v, 127)
    for k in (-6, -1, 3, 7):
        q2, s2 = orc.quantize_block(np.ldexp(v, k).astype(np.float32), 127)
        assert np.array_equal(q, q2)
        assert s2 == np.float32(np.ldexp(s, k))
    qn, sn = orc.quantize_block(-v, 127)
    assert np.array_equal(qn, -q) and sn == s
    # dequantise and quantise again: same codes; scale returns to within one fp32 step
    deq = (q.astype(np.float32) * s).astype(np.float32)
    q3, s3 = orc.quantize_block(deq, 127)
    assert np.array_equal(q3, q)
    assert abs(float(s3) - float(s)) <= float(s) * 2.0 ** -22


def test_zero_block_and_constant_block():
    q, s = orc.quantize_block(np.zeros(33, np.float32), 127)
    assert not q.any() and s == 0.0
    q, s = orc.quantize_block(np.full(17, -0.37, np.float32), 127)
    assert (q == -127).all()
    q, s = orc.quantize_block(np.full(17, 0.37, np.float32), 7)
    assert (q == 7).all()


def test_tokenwise_is_rowwise():
    rng = zq_inputs.rng_for(9, 3)
    y = rng.standard_normal((9, 48)).astype(np.float32)
    y[3] = 0
    y[5] *= 100
    xq, s = orc.quant_tokenwise(y)
    for m in range(9):
        q1, s1 = orc.quantize_block(y[m], 127)
        assert np.array_equal(xq[m], q1) and s[m] == s1
    assert s[3] == 0 and not xq[3].any()
    assert np.all(np.abs(xq).max(axis=1)[[0, 1, 2, 4, 5, 6, 7, 8]] == 127)


def test_group_geometry_is_blocks_of_output_rows():
    # group j = rows [j*gs, (j+1)*gs) over all K: give each row-block its own magnitude.
    N, K, g = 12, 8, 3
    w = np.zeros((N, K), np.float16)
    for j in range(g):
        w[j * 4:(j + 1) * 4, :] = np.float16(0.25 * (j + 1))
        w[j * 4, 0] = np.float16(2.0 ** j)          # the group's absmax
    wq, s_w, codes = orc.quantize_weight_groupwise(w, g, 8)
    for j in range(g):
        assert abs(float(s_w[j]) - 2.0 ** j / 127) <= 2.0 ** j / 127 * 2.0 ** -23
        assert codes[j * 4, 0] == 127
        want = _rne_fraction(Fraction(0.25 * (j + 1)) * 127 / Fraction(2.0 ** j))
        assert (codes[j * 4 + 1:(j + 1) * 4, :] == want).all()
    assert np.array_equal(wq, codes)
    # column blocks would give every group the same scale; it does not
    assert len(set(s_w.tolist())) == g


def test_groupwise_equals_blockwise_quantizer_on_random_weights():
    rng = zq_inputs.rng_for(9, 4)
    w = zq_inputs.weights(rng, 96, 64)
    for bits, qmax in ((8, 127), (4, 7)):
        wq, s_w, codes = orc.quantize_weight_groupwise(w, 6, bits)
        for j in range(6):
            blk = w[j * 16:(j + 1) * 16].astype(np.float32).reshape(-1)
            q, s = orc.quantize_block(blk, qmax)
            assert np.array_equal(codes[j * 16:(j + 1) * 16].reshape(-1), q)
            assert s_w[j] == s
        assert np.abs(codes).max() == qmax


def test_int4_nibble_order_and_roundtrip():
    # codes (1, -2) -> low nibble 0x1, high nibble 0xE
    w = np.array([[1.0, -2.0, 7.0, -7.0]], np.float16)
    wq, s_w, codes = orc.quantize_weight_groupwise(w, 1, 4)
    assert codes.tolist() == [[1, -2, 7, -7]]
    assert wq.tolist() == [[0xE1, 0x97]]
    assert s_w[0] == np.float32(1.0)
    # every byte value: unpack against sign-extension written with Python ints
    allb = np.arange(256, dtype=np.uint8)
    got = orc.unpack_int4(allb).reshape(256, 2)
    for b in range(256):
        lo, hi = b & 15, b >> 4
        assert got[b, 0] == (lo - 16 if lo > 7 else lo)
        assert got[b, 1] == (hi - 16 if hi > 7 else hi)
    # pack -> unpack returns the codes
    rng = zq_inputs.rng_for(9, 5)
    w = zq_inputs.weights(rng, 32, 64)
    wq, s_w, codes = orc.quantize_weight_groupwise(w, 2, 4)
    assert wq.shape == (32, 32)
    assert np.array_equal(orc.unpack_int4(wq), codes)
    assert codes.min() >= -7 and codes.max() <= 7


def test_groupwise_rejects_bad_arguments():
    w = np.zeros((10, 8), np.float16)
    with pytest.raises(ValueError):
        orc.quantize_weight_groupwise(w, 3, 8)
    with pytest.raises(ValueError):
        orc.quantize_weight_groupwise(w, 2, 5)


def test_oracle_matches_its_frozen_small_case():
    """tests/golden/quantizer_small.txt was written by tests/golden/make_quantizer_golden.py from
    oracle/ alone; the paper prints no worked example, so this only guards against unnoticed
    changes to the oracle's arithmetic."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_quantizer_golden", os.path.join(here, "make_quantizer_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(here, "quantizer_small.txt")) as f:
        stored = f.read().splitlines()
    assert stored == mod.lines()
