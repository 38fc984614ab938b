"""Host-only checks of the C ABI: the library loads without a GPU, exports every
symbol the header declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

import paper_2206_01861_amd as zq
from paper_2206_01861_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x10000  # a non-NULL, 16-byte aligned fake device address; never dereferenced on an error path
OK, E_NULL, E_SHAPE, E_ALIGN, E_UNSUP = 0, 1, 2, 3, 4
FIXED = zq.WORKSPACE_FIXED_BYTES   # control words, arrival counters and exchange slots in front of the partial sums


def test_workspace_constant_matches_the_header():
    text = open(os.path.join(ROOT, "include", "zq.h")).read()
    assert int(re.search(r"#define ZQ_WORKSPACE_FIXED_BYTES (\d+)", text).group(1)) == FIXED
    assert FIXED == 256 + 8192 * 4 + (1 << 19) * 8


def _declared(header="zq.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = zq.lib()
    names = _declared()
    assert "zq_gemm_i8_dequant" in names and "zq_quantize_weight_groupwise" in names
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(binding.SYMBOLS)
    probes = _declared("zq_probe.h")
    assert set(probes) == set(binding.PROBE_SYMBOLS)
    for n in probes:
        assert hasattr(L, n), n
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["zq.h", "zq_probe.h"]


def test_probe_validation():
    rs, mf = zq.lib().zq_probe_read_stream, zq.lib().zq_probe_mfma_i8
    assert rs(None, 1024, P, None) == E_NULL and rs(P, 1024, None, None) == E_NULL
    assert rs(P, 1000, P, None) == E_SHAPE and rs(P, 0, P, None) == E_SHAPE
    assert rs(P + 4, 1024, P, None) == E_ALIGN
    assert mf(None, 8, 10, P, None) == E_NULL and mf(P, 0, 10, P, None) == E_SHAPE and mf(P, 8, 0, P, None) == E_SHAPE
    assert mf(P, 8, 10, P + 8, None) == E_ALIGN
    tt = zq.lib().zq_probe_mfma_i8_tile_traffic
    assert tt(None, 2 << 20, 8, 10, P, None) == E_NULL and tt(P, 2 << 20, 8, 10, None, None) == E_NULL
    assert tt(P, (2 << 20) - 16, 8, 10, P, None) == E_SHAPE and tt(P, 2 << 20, 0, 10, P, None) == E_SHAPE
    assert tt(P, 2 << 20, 8, 0, P, None) == E_SHAPE and tt(P + 4, 2 << 20, 8, 10, P, None) == E_ALIGN


def test_status_strings_and_version():
    L = zq.lib()
    assert zq.version() >= 100
    seen = set()
    for code in range(6):
        s = L.zq_status_string(code).decode()
        assert s and s not in seen
        seen.add(s)


def test_variant_table():
    names = [zq.gemm_variant_name(i) for i in range(9)]
    assert names[0] == "simple" and None in names
    # decode shapes go to a weight-streaming schedule, prefill shapes to a tiled one
    assert zq.gemm_variant_name(zq.gemm_choose_variant(1, 6144, 2048)).startswith("skinny")
    assert zq.gemm_variant_name(zq.gemm_choose_variant(4096, 4096, 1024)).startswith("tile")
    assert zq.gemm_variant_name(zq.gemm_choose_variant(128, 768, 784)) == "simple"   # tiny: untiled
    assert zq.gemm_variant_name(zq.gemm_choose_variant(4096, 768, 784)).startswith("tile")   # ragged K is tiled too
    ws = zq.gemm_workspace_bytes(64, 6144, 24576)
    assert ws > FIXED and (ws - FIXED) % (64 * 6144 * 4) == 0
    assert zq.gemm_variant_name(zq.gemm_choose_variant(64, 6144, 24576, 8, ws)) == "skinny_splitk"
    assert zq.gemm_variant_name(zq.gemm_choose_variant(64, 6144, 24576, 8, ws - 1)) == "skinny"
    assert zq.gemm_workspace_bytes(4096, 4096, 1024) == 0
    # 256-row tiles: 256 columns unless narrower tiles fill the 256 compute units better
    assert zq.gemm_variant_name(zq.gemm_choose_variant(4096, 4096, 1024)) == "tile256"       # 256 tiles: one round
    assert zq.gemm_variant_name(zq.gemm_choose_variant(2048, 6144, 2048)) == "tile256x192"   # 192 tiles -> 256
    assert zq.gemm_variant_name(zq.gemm_choose_variant(4096, 12288, 4096)) == "tile256"      # 768 tiles: three rounds
    assert zq.gemm_variant_name(zq.gemm_choose_variant(16384, 18432, 6144)) == "tile256"


def test_stream_plan_covers_the_matrix():
    """The cut of the weight-streaming schedules: every strip has a consumer wave, no split
    is empty, a K split is only planned when the offered workspace holds its partials."""
    import random
    rnd = random.Random(7)
    shapes = [(64, 6144, 24576, 8), (16, 4096, 16384, 4), (1, 768, 768, 8), (64, 18432, 6144, 8),
              (16, 196608, 4096, 4), (7, 16, 256, 8), (64, 131072, 256, 8)]
    for _ in range(200):
        shapes.append((rnd.randint(1, 128), 16 * rnd.randint(1, 3000), 256 * rnd.randint(1, 100), rnd.choice([4, 8])))
    for M, N, K, bits in shapes:
        ws = zq.gemm_workspace_bytes(M, N, K, bits)
        for offered in (0, ws):
            rb, ks, c = zq.gemm_stream_plan(M, N, K, bits, offered)
            strips, stages = N // 16, K // 256
            assert 1 <= rb <= strips and 1 <= ks <= stages and 1 <= c <= 8
            assert c == -(-strips // rb)                  # the fullest row block fits the workgroup
            if offered == 0:
                assert ks == 1
            elif ks > 1:                                  # (the workspace may also be another schedule's)
                assert ws >= ks * M * N * 4 and strips <= 8192
    with pytest.raises(zq.ZQError):
        zq.gemm_stream_plan(129, 1024, 1024)
    with pytest.raises(zq.ZQError):
        zq.gemm_stream_plan(8, 1024, 1000)


def test_stream_k_ranges_only_where_they_apply():
    """Two K ranges per strip: INT8 weights, at most 32 tokens, no K split, at least 4096 deep,
    and at most four strips per workgroup (two waves each, eight consumer waves at most)."""
    import random
    rnd = random.Random(11)
    assert zq.gemm_stream_k_ranges(1, 4096, 4096, 8, 0) == 2
    assert zq.gemm_stream_k_ranges(16, 12288, 4096, 8, 0) == 2
    assert zq.gemm_stream_k_ranges(1, 4096, 4096, 4, 0) == 1          # INT4 weights
    assert zq.gemm_stream_k_ranges(33, 4096, 4096, 8, 0) == 1         # more than two token tiles
    assert zq.gemm_stream_k_ranges(1, 4096, 2048, 8, 0) == 1          # K too short
    assert zq.gemm_stream_k_ranges(129, 4096, 4096, 8, 0) == 0 and zq.gemm_stream_k_ranges(1, 4096, 1000, 8, 0) == 0
    seen = 0
    for _ in range(300):
        M, N, K, bits = rnd.randint(1, 128), 16 * rnd.randint(1, 1500), 256 * rnd.randint(1, 100), rnd.choice([4, 8])
        ws = zq.gemm_workspace_bytes(M, N, K, bits)
        for offered in (0, ws):
            r = zq.gemm_stream_k_ranges(M, N, K, bits, offered)
            rb, ks, c = zq.gemm_stream_plan(M, N, K, bits, offered)
            assert r in (1, 2)
            if r == 2:
                seen += 1
                assert bits == 8 and M <= 32 and ks == 1 and K >= 4096 and c <= 4 and N <= 3 * 256 * 16
    assert seen > 0


def test_weight_quant_validation():
    f = zq.lib().zq_quantize_weight_groupwise
    assert f(None, 64, 64, 4, 8, P, P, None) == E_NULL
    assert f(P, 64, 64, 4, 8, None, P, None) == E_NULL
    assert f(P, 64, 64, 4, 5, P, P, None) == E_UNSUP
    assert f(P, 0, 64, 4, 8, P, P, None) == E_SHAPE
    assert f(P, 64, 64, 3, 8, P, P, None) == E_SHAPE        # N % g
    assert f(P, 64, 64, 8, 8, P, P, None) == E_SHAPE        # group of 8 rows
    assert f(P, 64, 40, 4, 8, P, P, None) == E_SHAPE        # K % 16
    assert f(P, 64, 48, 4, 4, P, P, None) == E_SHAPE        # K % 32 for INT4
    assert f(P + 4, 64, 64, 4, 8, P, P, None) == E_ALIGN


def test_rowquant_validation():
    ln = zq.lib().zq_layernorm_quant_tokenwise
    ge = zq.lib().zq_gelu_quant_tokenwise
    assert ln(None, P, P, 1e-5, 4, 64, P, P, None, 0, None) == E_NULL
    assert ln(P, None, P, 1e-5, 4, 64, P, P, None, 0, None) == E_NULL      # gamma is required
    assert ln(P, P, None, 1e-5, 4, 60, P, P, None, 0, None) == E_SHAPE
    assert ln(P, P, None, 1e-5, 0, 64, P, P, None, 0, None) == E_SHAPE
    assert ln(P, P, None, 1e-5, 4, 65536, P, P, None, 0, None) == E_SHAPE
    assert ln(P, P, None, 1e-5, 4, 64, P, P, P, 2, None) == E_UNSUP
    assert ln(P, P, None, -1.0, 4, 64, P, P, None, 0, None) == E_UNSUP
    assert ln(P, P, None, 1e-5, 4, 64, P + 8, P, None, 0, None) == E_ALIGN
    assert ge(P, None, 0, 4, 64, None, P, None, 0, None) == E_NULL
    assert ge(P, None, 2, 4, 64, P, P, None, 0, None) == E_UNSUP
    assert ge(P, None, 0, 4, 72, P, P, None, 0, None) == E_SHAPE


@pytest.mark.parametrize("fname,kmul", [("zq_gemm_i8_dequant", 16), ("zq_gemm_w4a8_dequant", 32)])
def test_gemm_validation(fname, kmul):
    f = getattr(zq.lib(), fname)

    def call(xq=P, s_tok=P, wq=P, s_w=P, groups=4, bias=None, M=8, N=64, K=128, out=P, acc=None,
             out_q=None, out_s=None, ws=None, ws_bytes=0):
        return f(xq, s_tok, wq, s_w, groups, bias, M, N, K, out, acc, out_q, out_s, ws, ws_bytes, None)

    assert call(xq=None) == E_NULL
    assert call(out=None) == E_NULL
    assert call(out_q=P) == E_NULL                 # re-quantization outputs come as a pair
    assert call(M=0) == E_SHAPE
    assert call(groups=3) == E_SHAPE
    assert call(groups=8) == E_SHAPE               # 8 columns per group
    assert call(K=128 + kmul // 2) == E_SHAPE
    assert call(K=133152) == E_SHAPE               # INT32 accumulator could wrap
    if kmul == 32:                                 # INT4 codes travel as code * 16 and -8 is legal: K * 127 * 128 < 2^31
        assert call(K=132128) == E_SHAPE
        prev = zq.force_gemm_variant(3)
        try:
            assert call(K=132064) == E_UNSUP       # inside the bound: refused only by the forced schedule, nothing launched
        finally:
            zq.force_gemm_variant(prev)
    assert call(M=65536, K=32768) == E_SHAPE       # an operand of 2 GiB: beyond the 32-bit buffer offsets
    assert call(N=65536 * (2 if kmul == 32 else 1), K=32768, groups=64) == E_SHAPE
    assert call(bias=P + 2) == E_ALIGN
    prev = zq.force_gemm_variant(3)
    try:
        assert call(K=kmul * 3) == E_UNSUP         # forced streaming schedule steps K by 256: nothing is launched
    finally:
        zq.force_gemm_variant(prev)
    assert zq.force_gemm_variant(-1) == -1


def test_gemm_gelu_quant_validation():
    f = zq.lib().zq_gemm_gelu_quant_tokenwise

    def call(xq=P, s_tok=P, wq=P, w_bits=8, s_w=P, groups=4, bias=None, tanh=0, M=8, N=64, K=128, g=P, gq=P, s=P):
        return f(xq, s_tok, wq, w_bits, s_w, groups, bias, tanh, M, N, K, g, gq, s, None, 0, None)

    assert call(w_bits=5) == E_UNSUP
    assert call(tanh=2) == E_UNSUP
    assert call(gq=None) == E_NULL
    assert call(s=None) == E_NULL
    # eight tokens run on a streaming schedule, whose output a second kernel quantizes: that kernel
    # reads the FP16 tensor, so the call is refused without it (nothing is launched)
    assert zq.lib().zq_gemm_quantizes_in_kernel(8, 64, 128, 8, 0) == 0
    assert call(g=None) == E_UNSUP
    assert call(wq=None) == E_NULL
    assert call(N=32768 + 64, groups=4) == E_SHAPE # a row of g must fit the quantizer's registers
    assert call(K=48, w_bits=4) == E_SHAPE
    assert call(g=P + 8) == E_ALIGN


def test_where_the_output_is_quantized():
    """Tiled schedules quantize in the GeMM kernel, within the limits of the exchange arrays and of
    the band that must be resident at once; the debug switch turns it off."""
    q = zq.gemm_quantizes_in_kernel
    def q(M, N, K, bits, ws=FIXED):
        return zq.gemm_quantizes_in_kernel(M, N, K, bits, ws)

    assert q(4096, 4096, 1024, 8) and q(4096, 4096, 1024, 4) and q(16384, 6144, 24576, 8)
    assert not q(4096, 4096, 1024, 8, 0) and not q(4096, 4096, 1024, 8, FIXED - 1)   # the exchange lives in the workspace
    assert q(32768, 4096, 64, 8) and not q(32769, 4096, 64, 8)            # exchange slots of a workspace
    assert q(4096, 16384, 4096, 8) and not q(4096, 16384 + 256, 4096, 8)  # tiles per band: a quarter of 256 compute units
    assert not q(64, 4096, 4096, 8) and not q(1, 16, 16, 8)               # streaming / untiled schedules
    assert not q(0, 16, 16, 8) and not q(16, 16, 16, 5)
    prev = zq.set_in_kernel_quant(False)
    try:
        assert prev is True and not q(4096, 4096, 1024, 8)
    finally:
        assert zq.set_in_kernel_quant(prev) is False
    assert q(4096, 4096, 1024, 8)
    # the size query for calls with quantized output: the fixed part where the kernel quantizes, and never
    # less than the plain call's
    assert zq.gemm_quant_workspace_bytes(4096, 4096, 1024, 8) == FIXED and zq.gemm_workspace_bytes(4096, 4096, 1024, 8) == 0
    assert zq.gemm_quant_workspace_bytes(8, 256, 256, 8) == 0
    assert zq.gemm_quant_workspace_bytes(32, 2048, 8192, 8) == zq.gemm_workspace_bytes(32, 2048, 8192, 8) > FIXED
    assert zq.gemm_quant_workspace_bytes(192, 4096, 4096, 8) == zq.gemm_workspace_bytes(192, 4096, 4096, 8)
    c = ctypes.c_int(0)
    assert zq.lib().zq_quant_wait_expired(None, ctypes.byref(c)) == E_NULL
    assert zq.lib().zq_quant_wait_expired(P, None) == E_NULL
    assert zq.lib().zq_quant_wait_expired(P + 4, ctypes.byref(c)) == E_ALIGN


def test_workspace_init_validation():
    f = zq.lib().zq_workspace_init
    assert f(None, FIXED, None) == E_NULL
    assert f(P, FIXED - 1, None) == E_SHAPE
    assert f(P, 0, None) == E_SHAPE
    assert f(P + 8, FIXED, None) == E_ALIGN


def test_standalone_quantizer_and_dequantizer_validation():
    q = zq.lib().zq_quantize_tokenwise
    assert q(None, 4, 64, P, P, None) == E_NULL
    assert q(P, 4, 64, None, P, None) == E_NULL
    assert q(P, 0, 64, P, P, None) == E_SHAPE
    assert q(P, 4, 72, P, P, None) == E_SHAPE
    assert q(P, 4, 32768 + 16, P, P, None) == E_SHAPE
    assert q(P + 4, 4, 64, P, P, None) == E_ALIGN
    d = zq.lib().zq_dequantize_acc
    assert d(None, P, P, 4, None, 8, 64, P, None) == E_NULL
    assert d(P, P, P, 4, None, 8, 64, None, None) == E_NULL
    assert d(P, P, P, 3, None, 8, 64, P, None) == E_SHAPE
    assert d(P, P, P, 8, None, 8, 64, P, None) == E_SHAPE          # 8 columns per group
    assert d(P, P, P, 4, None, 0, 64, P, None) == E_SHAPE
    assert d(P, P, P, 4, P + 2, 8, 64, P, None) == E_ALIGN


def test_tuning_table_overrides_the_choice():
    zq.tune_clear()
    try:
        M, N, K = 16, 4096, 4096
        base = zq.gemm_choose_variant(M, N, K, 8, 0)
        assert zq.gemm_variant_name(base) == "skinny"
        zq.tune_set(1, 32, N, K, 8, 1)                              # 128x128 tiles for 1..32 tokens
        assert zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, 8, 0)) == "tile128"
        assert zq.gemm_choose_variant(33, N, K, 8, 0) == zq.gemm_choose_variant(33, N, K, 4, 0)   # outside the range
        assert zq.gemm_choose_variant(M, N, K, 4, 0) == base        # other bit width untouched
        # a streaming cut with a K split: the workspace query and the plan follow it
        zq.tune_set(1, 32, N, K, 8, 4, 64, 4)
        ws = zq.gemm_workspace_bytes(M, N, K, 8)
        assert ws == FIXED + 4 * M * N * 4
        assert zq.gemm_stream_plan(M, N, K, 8, ws) == (64, 4, 4)
        assert zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, 8, ws)) == "skinny_splitk"
        assert zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, 8, 0)) == "skinny"   # no workspace: entry ignored
        assert zq.gemm_stream_plan(M, N, K, 8, 0)[1] == 1
        assert zq.tune_count() == 2
        for bad in ((1, 32, N, K, 8, 3, 16, 1),      # 16 strips per row block: more than a workgroup has waves
                    (1, 32, N, K, 8, 3, 64, 4),      # a K split belongs to the split schedule
                    (1, 32, N, K, 8, 4, 64, 17),     # more splits than stages
                    (32, 1, N, K, 8, 1, 0, 0), (1, 32, N, K, 5, 1, 0, 0)):
            with pytest.raises(zq.ZQError):
                zq.tune_set(*bad)
        with pytest.raises(zq.ZQError):
            zq.tune_set(1, 32, N, K, 8, 9)
        with pytest.raises(zq.ZQError):
            zq.tune_set(1, 32, N, K, 8, 1, 64, 1)    # a cut for a tiled schedule
    finally:
        zq.tune_clear()
    assert zq.tune_count() == 0 and zq.gemm_choose_variant(16, 4096, 4096, 8, 0) == base


def test_tile_k_split_dispatch():
    """Above the streaming schedules' token counts, a shape whose 128x128 tiles would occupy less than
    half the chip splits K when the workspace holds the partial products, and only then."""
    for (M, N, K) in [(192, 4096, 4096), (300, 2048, 8192), (130, 4096, 4000), (96, 1040, 3968)]:
        ws = zq.gemm_workspace_bytes(M, N, K, 8)
        assert ws > FIXED and (ws - FIXED) % (M * N * 4) == 0 and 2 <= (ws - FIXED) // (M * N * 4) <= 16
        assert zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, 8, ws)) == "tile128_splitk"
        assert zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, 8, ws - 1)) != "tile128_splitk"
        assert zq.gemm_workspace_bytes(M, N, K, 4) == ws            # the INT4 call splits alike
    for (M, N, K) in [(1024, 4096, 4096), (384, 4096, 4096), (256, 4096, 1024), (4096, 4096, 1024), (129, 12288, 4096)]:
        assert zq.gemm_workspace_bytes(M, N, K, 8) == 0             # enough tiles, or K too short to pay
    # 65 to 128 tokens: the K split where K is long, streaming otherwise and always up to 64 tokens
    assert zq.gemm_variant_name(zq.gemm_choose_variant(100, 4096, 4096, 8, 1 << 30)) == "tile128_splitk"
    assert zq.gemm_variant_name(zq.gemm_choose_variant(100, 4096, 4096, 8, 0)) == "skinny"
    assert zq.gemm_variant_name(zq.gemm_choose_variant(100, 2048, 2048, 8, 1 << 30)) == "skinny"
    assert zq.gemm_variant_name(zq.gemm_choose_variant(64, 4096, 4096, 8, 1 << 30)) == "skinny"


def test_w8a16_validation():
    f = zq.lib().zq_gemm_w8a16_dequant

    def call(x=P, wq=P, s_w=P, groups=4, bias=None, M=8, N=64, K=128, out=P, ws=None, ws_bytes=0):
        return f(x, wq, s_w, groups, bias, M, N, K, out, ws, ws_bytes, None)

    assert call(x=None) == E_NULL
    assert call(wq=None) == E_NULL
    assert call(out=None) == E_NULL
    assert call(M=0) == E_SHAPE
    assert call(groups=3) == E_SHAPE
    assert call(K=136) == E_SHAPE
    assert call(K=133152) == E_SHAPE
    assert call(x=P + 2) == E_ALIGN
    assert call(ws=P + 4, ws_bytes=64) == E_ALIGN


def test_w8a16_workspace_and_plan():
    """The W8A16 call's own workspace query: the size of the fp32 partials of the cut it would take
    (for 65 to 128 tokens, of its 64-token launches), 0 where it never splits; the plan covers the matrix."""
    for (M, N, K) in [(1, 2048, 8192), (32, 2048, 8192), (64, 6144, 24576), (16, 12288, 4096), (64, 4112, 16384)]:
        ws = zq.gemm_w8a16_workspace_bytes(M, N, K)
        rb, ks, c = zq.gemm_w8a16_stream_plan(M, N, K, ws)
        assert 1 <= rb <= N // 16 and 1 <= c <= 8 and c == -(-(N // 16) // rb)
        assert ws == (FIXED + ks * M * N * 4 if ks > 1 else 0)
        assert zq.gemm_w8a16_stream_plan(M, N, K, 0)[1] == 1
    # 65 to 128 tokens: at least what the 64-token streaming launches need, more where the tiled schedule
    # with a K split is the faster choice
    assert zq.gemm_w8a16_workspace_bytes(100, 2048, 8192) >= zq.gemm_w8a16_workspace_bytes(64, 2048, 8192) > 0
    assert zq.gemm_w8a16_workspace_bytes(100, 18432, 6144) == zq.gemm_w8a16_workspace_bytes(64, 18432, 6144)
    # above 128 tokens: the tiled schedule, which splits K where its tiles would leave most of the chip idle
    assert (zq.gemm_w8a16_workspace_bytes(129, 2048, 8192) - FIXED) % (129 * 2048 * 4) == 0
    assert zq.gemm_w8a16_workspace_bytes(129, 2048, 8192) >= FIXED + 2 * 129 * 2048 * 4
    assert zq.gemm_w8a16_workspace_bytes(4096, 4096, 4096) == 0
    assert zq.gemm_w8a16_workspace_bytes(16, 2048, 1000) == 0       # K not a multiple of 256: untiled
    with pytest.raises(zq.ZQError):
        zq.gemm_w8a16_stream_plan(65, 2048, 8192)


def test_missing_library_is_an_error(tmp_path, monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libzq.so"))
    with pytest.raises(ImportError):
        binding.lib()
