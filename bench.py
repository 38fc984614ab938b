#!/usr/bin/env python3
"""Benchmark of the quantized linear layer on one MI355X.

Default run (`python bench.py`): the BERT-large feed-forward pair of the
paper's BERT-large workload (batch 32 x sequence 128 = 4096 tokens),
  LayerNorm+quant -> INT8 GeMM 1024->4096 (+bias) -> GeLU+quant -> INT8 GeMM 4096->1024 (+bias),
with inputs resident in HBM.  A step is one pass of that chain.  The chain is
captured once into a HIP graph and replayed (the paper replays a CUDA graph for
both its INT8 and its FP16 runs, App. D); the FP16 comparator is captured the
same way.  Prints ONE JSON line: whole-chain throughput in TOPS, the roofline
of the dominant kernel (the tiled INT8 GeMM, launched twice per step), the
same chain in FP16 through torch (hipBLASLt / rocBLAS), the CPU oracle timed
on the host cores, and a `rows` array with the GeMMs the roofline targets are
stated on: the largest prefill shapes (against the INT8 matrix-core peak) and
decode shapes whose weight buffers rotate through more than 512 MB (against
the HBM peak), each the median of five repeats of at least fifty launches,
with the oracle timed beside it.

`python bench.py --table` instead times every linear of every workload shape
(prefill: TOPS against the INT8 matrix-core peak; decode: GB/s against HBM,
with buffers rotated through more than 512 MB so the Infinity Cache cannot
serve them), writes the rows as JSON to the file given by --table-json and prints the table to stderr.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import zq_inputs  # noqa: E402

PEAK_INT8_TOPS = 5000.0    # MI355X dense INT8 matrix-core peak, TOP/s
PEAK_HBM_GBS = 8000.0
# HBM-side bytes one tiled-GeMM launch of the default workload moves, mean of the two launches of a
# step: rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a 256 MiB copy.  A constant taken from the
# profile named below, not measured in this run (algorithmic bytes are 40 MiB and 28 MiB).
GEMM_TRAFFIC_BYTES = 56.3 * (1 << 20)
GEMM_TRAFFIC_SOURCE = "profiles/c2_ffc_pair_hbm_traffic.txt"
ROTATE_BYTES = 640 << 20   # decode rows: operands rotate through more than twice the 256 MB Infinity Cache
# GeMMs reported next to the headline: (linear, tokens, bound)
ROWS = [("c5_ffc1", 16384, "mfma"), ("c4_qkv", 4096, "mfma"), ("c5_ffc1", 64, "hbm"), ("c4_ffc1", 1, "hbm"),
        ("c4_qkv", 1, "hbm"), ("c4_qkv", 16, "hbm")]


def _events(n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def graph_of(fn, reps):
    """Capture `reps` calls of fn(i) on a side stream into one HIP graph."""
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        for i in range(min(reps, 3)):
            fn(i)                      # warm up outside the capture (lazy module load, attributes)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(reps):
            fn(i)
    return g


class ClockSampler:
    """Reads the shader clock from sysfs on a host thread while the GPU works; .mhz is the median of the
    samples taken, or None where the file is not readable or the region was too short for a sample."""

    def __init__(self):
        self.samples, self._stop, self._thread, self.mhz = [], False, None, None

    def _run(self):
        while not self._stop:
            v = sclk_mhz()
            if v is None:
                return
            self.samples.append(v)
            time.sleep(0.0005)

    def __enter__(self):
        import threading
        self._thread = threading.Thread(target=self._run, daemon=True)
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        self._thread.join()
        if self.samples:
            self.mhz = float(np.median(self.samples))


def time_graph_median(g, reps_per_replay, repeats=5, warm=1, clock=None):
    """Median over `repeats` timed replays of a graph of `reps_per_replay` calls: ms per call.
    clock: a dict that receives "sclk_mhz", the median shader clock sampled while the replays ran."""
    for _ in range(warm):
        g.replay()
    torch.cuda.synchronize()
    times = []
    with ClockSampler() as cs:
        for _ in range(repeats):
            e0, e1 = _events(2)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) / reps_per_replay)
    if clock is not None:
        clock["sclk_mhz"] = cs.mhz
    return float(np.median(times))


def sclk_mhz():
    """The shader clock the driver reports right now (sysfs), or None where it is not readable."""
    import glob
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        try:
            for line in open(path):
                if "*" in line:
                    return float(line.split(":")[1].replace("*", "").strip().lower().replace("mhz", ""))
        except (OSError, ValueError, IndexError):
            continue
    return None


def time_graph(g, replays, reps_per_replay, warm=2):
    for _ in range(warm):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = _events(2)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * reps_per_replay)      # ms per call


class FFCPair:
    """Workload c2: tensors resident on the GPU, weights quantized once (the offline step)."""

    def __init__(self, zq, tokens=4096, hidden=1024, ffn=4096, groups=64):
        self.zq = zq
        self.M, self.H, self.F, self.g = tokens, hidden, ffn, groups
        rng = zq_inputs.rng_for(2, 0)
        self.x_h = zq_inputs.config_activations("c2", rng, tokens, hidden)
        self.gamma_h, self.beta_h = zq_inputs.layernorm_params(rng, hidden)
        self.w1_h, self.b1_h = zq_inputs.weights(rng, ffn, hidden), zq_inputs.bias(rng, ffn)
        self.w2_h, self.b2_h = zq_inputs.weights(rng, hidden, ffn), zq_inputs.bias(rng, hidden)
        self.x, self.gamma, self.beta = _dev(self.x_h), _dev(self.gamma_h), _dev(self.beta_h)
        self.w1, self.b1, self.w2, self.b2 = _dev(self.w1_h), _dev(self.b1_h), _dev(self.w2_h), _dev(self.b2_h)
        zq.zq_quantize_weight_groupwise(self.w1, groups, 8)      # warm
        torch.cuda.synchronize()
        t0, t1 = _events(2)
        t0.record()
        self.wq1, self.sw1 = zq.zq_quantize_weight_groupwise(self.w1, groups, 8)
        self.wq2, self.sw2 = zq.zq_quantize_weight_groupwise(self.w2, groups, 8)
        t1.record()
        torch.cuda.synchronize()
        self.weight_quant_ms = t0.elapsed_time(t1)
        d = "cuda"
        self.xq = torch.empty((tokens, hidden), dtype=torch.int8, device=d)
        self.st = torch.empty(tokens, dtype=torch.float32, device=d)
        self.h = torch.empty((tokens, ffn), dtype=torch.float16, device=d)
        self.hq = torch.empty((tokens, ffn), dtype=torch.int8, device=d)
        self.st2 = torch.empty(tokens, dtype=torch.float32, device=d)
        self.o = torch.empty((tokens, hidden), dtype=torch.float16, device=d)
        self.acc1 = torch.empty((tokens, ffn), dtype=torch.int32, device=d)      # only the unfused ablation uses these
        self.acc2 = torch.empty((tokens, hidden), dtype=torch.int32, device=d)
        # workspace of the fused call: its GeMM kernel exchanges row maxima through it
        self.ws = zq.new_workspace(zq.gemm_quant_workspace_bytes(tokens, ffn, hidden, 8))
        self.ops = 2.0 * tokens * (hidden * ffn + ffn * hidden)
        self.gemm_ops = 2.0 * tokens * hidden * ffn          # per GeMM launch (both are equal)

    def ln(self, _=0):
        self.zq.zq_layernorm_quant_tokenwise(self.x, self.gamma, self.beta, 1e-5, out=(self.xq, self.st))

    def gemm1(self, _=0):
        self.zq.zq_gemm_i8_dequant(self.xq, self.st, self.wq1, self.sw1, self.b1, out=self.h)

    def gelu(self, _=0):
        self.zq.zq_gelu_quant_tokenwise(self.h, None, out=(self.hq, self.st2))

    def gemm2(self, _=0):
        self.zq.zq_gemm_i8_dequant(self.hq, self.st2, self.wq2, self.sw2, self.b2, out=self.o)

    def step(self, _=0):
        self.ln()
        self.gemm1()
        self.gelu()
        self.gemm2()

    def gemm1_gelu(self, _=0):
        """GeMM 1 with bias + GeLU + token-wise quantization inside the GeMM kernel; the FP16 activation
        is never written (the second GeMM only reads the codes)."""
        self.zq.zq_gemm_gelu_quant_tokenwise(self.xq, self.st, self.wq1, self.sw1, self.b1,
                                             out=(None, self.hq, self.st2), keep_g=False, workspace=self.ws)

    def gemm1_gelu_keep(self, _=0):
        self.zq.zq_gemm_gelu_quant_tokenwise(self.xq, self.st, self.wq1, self.sw1, self.b1,
                                             out=(self.h, self.hq, self.st2), workspace=self.ws)

    def fused_step(self, _=0):
        """Same layer with bias + GeLU in the epilogue of the first GeMM (three calls instead of four)."""
        self.ln()
        self.gemm1_gelu()
        self.gemm2()

    def unfused_step(self, _=0):
        """The pipeline the fusions replace (Fig. 2, left): FP16 LayerNorm and GeLU as kernels of their own
        (torch), a separate quantization kernel, a GeMM that writes its INT32 accumulators to memory and a
        separate dequantization kernel.  (The GeMM call also writes its FP16 output, which this chain ignores.)"""
        F = torch.nn.functional
        zq = self.zq
        y = F.layer_norm(self.x, (self.H,), self.gamma, self.beta, 1e-5)
        zq.zq_quantize_tokenwise(y, out=(self.xq, self.st))
        zq.zq_gemm_i8_dequant(self.xq, self.st, self.wq1, self.sw1, None, out=self.h, acc_out=self.acc1)
        zq.zq_dequantize_acc(self.acc1, self.st, self.sw1, self.b1, out=self.h)
        a = F.gelu(self.h)
        zq.zq_quantize_tokenwise(a, out=(self.hq, self.st2))
        zq.zq_gemm_i8_dequant(self.hq, self.st2, self.wq2, self.sw2, None, out=self.o, acc_out=self.acc2)
        zq.zq_dequantize_acc(self.acc2, self.st2, self.sw2, self.b2, out=self.o)

    def fp16_step(self, _=0):
        F = torch.nn.functional
        y = F.layer_norm(self.x, (self.H,), self.gamma, self.beta, 1e-5)
        h = F.linear(y, self.w1, self.b1)
        a = F.gelu(h)
        return F.linear(a, self.w2, self.b2)


def cpu_baseline(wl):
    """The oracle, as it stands, on the host cores, over the same chain and the same tokens."""
    from oracle import zq_oracle as orc
    wq1, sw1, _ = orc.quantize_weight_groupwise(wl.w1_h, wl.g, 8)
    wq2, sw2, _ = orc.quantize_weight_groupwise(wl.w2_h, wl.g, 8)
    t0 = time.perf_counter()
    _, y32 = orc.layernorm(wl.x_h, wl.gamma_h, wl.beta_h, 1e-5)
    xq, st = orc.quant_tokenwise(y32)
    acc = orc.matmul_i32(xq, wq1)
    ref, _ = orc.dequant(acc, st, sw1, wl.b1_h)
    h16 = ref.astype(np.float16)
    _, g32 = orc.gelu(h16, None)
    hq, st2 = orc.quant_tokenwise(g32)
    acc2 = orc.matmul_i32(hq, wq2)
    orc.dequant(acc2, st2, sw2, wl.b2_h)
    dt = time.perf_counter() - t0
    return {"value": wl.ops / dt / 1e12, "unit": "TOPS", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "one step of the same chain, all %d tokens, %.2f s wall" % (wl.M, dt)}


def measured_ceilings(zq):
    """What the installed part sustains, next to the datasheet peaks (include/zq_probe.h): a read-only
    stream over 1.25 GB, and the INT8 matrix cores alone on register operands of three kinds."""
    res = {}
    buf = torch.empty(1280 << 20, dtype=torch.uint8, device="cuda").random_(0, 256)
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    g = graph_of(lambda i: zq.zq_probe_read_stream(buf, sink), 10)
    ms = time_graph_median(g, 10)
    res["hbm_read_stream_GBs"] = buf.numel() / (ms * 1e-3) / 1e9
    del buf, g
    torch.cuda.empty_cache()
    blocks, iters = 512, 1500                      # two workgroups of four waves per compute unit
    nbytes = blocks * 256 * 128
    out = torch.empty(blocks * 256 * 16, dtype=torch.uint8, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(zq_inputs.BASE_SEED % (2 ** 31))
    xq, _ = _codes(gen, nbytes // 2 // 4096, 4096, "c5")             # token-wise codes of N(0,1) rows
    w = torch.randn((nbytes // 2 // 4096, 4096), generator=gen, device="cuda")
    wq = torch.round(w * (127.0 / w.abs().amax())).to(torch.int8)      # one weight group
    kinds = {"uniform_random_bytes": torch.randint(0, 256, (nbytes,), generator=gen, device="cuda", dtype=torch.uint8),
             "workload_codes": torch.cat([xq.view(torch.uint8).flatten(), wq.view(torch.uint8).flatten()]),
             "zero_operands": torch.zeros(nbytes, dtype=torch.uint8, device="cuda")}
    for kind, ops_buf in kinds.items():
        clk = {}
        nops = [0]

        def run(i, ops_buf=ops_buf):
            nops[0] = zq.zq_probe_mfma_i8(ops_buf, blocks, iters, out)
        g = graph_of(run, 5)
        ms = time_graph_median(g, 5, clock=clk)
        res["mfma_i8_TOPS_" + kind] = nops[0] / (ms * 1e-3) / 1e12
        res["mfma_i8_sclk_mhz_" + kind] = clk.get("sclk_mhz")
    # the same matrix-core stream with the operand traffic of the 256x256 tile (LDS fragment reads and
    # global -> LDS stages, no barriers, prologue or epilogue): the ceiling of that tile design on this part
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out2 = torch.empty(cus * 512 * 16, dtype=torch.uint8, device="cuda")
    for kind in ("uniform_random_bytes", "workload_codes"):
        nops = [0]

        src2 = kinds[kind]
        if kind == "workload_codes":                # the 2 MiB window the probe reads: half activation codes, half weight codes
            src2 = torch.cat([xq.view(torch.uint8).flatten()[:1 << 20], wq.view(torch.uint8).flatten()[:1 << 20]])

        def run2(i, src=src2):
            nops[0] = zq.zq_probe_mfma_i8_tile_traffic(src, cus, 1500, out2)
        g = graph_of(run2, 5)
        ms = time_graph_median(g, 5)
        res["mfma_i8_TOPS_with_tile_traffic_" + kind] = nops[0] / (ms * 1e-3) / 1e12
    res["note"] = ("matrix cores alone: 512 workgroups x 4 waves, 16 accumulators per wave, operands in registers; the "
                   "clock, and with it the figure, follows the power the operand bytes make the multipliers draw. "
                   "with_tile_traffic: one workgroup of eight waves per compute unit, every wave the 128x64 wave tile of "
                   "the 256x256 schedule with its LDS fragment reads and its global->LDS stage loads, without barriers, "
                   "prologue or epilogue")
    return res


def rotated_frontends(zq, wl):
    """LayerNorm+quant and GeLU+quant of the workload with inputs and outputs rotating through more
    than 512 MB, so that neither the reads nor the writes are served by the Infinity Cache."""
    M, H, F = wl.M, wl.H, wl.F
    res = {}
    n_ln = -(-ROTATE_BYTES // (3 * M * H))
    xs = [torch.randn((M, H), device="cuda").half() for _ in range(n_ln)]
    qs = [torch.empty((M, H), dtype=torch.int8, device="cuda") for _ in range(n_ln)]
    reps = -(-50 // n_ln) * n_ln
    g = graph_of(lambda i: zq.zq_layernorm_quant_tokenwise(xs[i % n_ln], wl.gamma, wl.beta, 1e-5,
                                                           out=(qs[i % n_ln], wl.st)), reps)
    us = time_graph_median(g, reps) * 1e3
    res["layernorm_quant"] = {"us": us, "GBs": (3.0 * M * H + 4 * H + 4 * M) / (us * 1e-6) / 1e9, "sets": n_ln}
    del xs, qs, g
    n_g = -(-ROTATE_BYTES // (3 * M * F))
    hs = [torch.randn((M, F), device="cuda").half() for _ in range(n_g)]
    qs = [torch.empty((M, F), dtype=torch.int8, device="cuda") for _ in range(n_g)]
    reps = -(-50 // n_g) * n_g
    g = graph_of(lambda i: zq.zq_gelu_quant_tokenwise(hs[i % n_g], None, out=(qs[i % n_g], wl.st2)), reps)
    us = time_graph_median(g, reps) * 1e3
    res["gelu_quant"] = {"us": us, "GBs": (3.0 * M * F + 4 * M) / (us * 1e-6) / 1e9, "sets": n_g}
    return res


def c1_chain(zq):
    """Workload c1 (one BERT-base linear at 128 tokens) as the chain LayerNorm+quant -> GeMM 768 -> 768:
    HIP-graph replay against launching the two calls one by one (App. D: on small models the launches
    cost more than the kernels)."""
    rng = zq_inputs.rng_for(1, 0)
    M, H, g = 128, 768, 48
    x = _dev(zq_inputs.config_activations("c1", rng, M, H))
    gamma_h, beta_h = zq_inputs.layernorm_params(rng, H)
    gamma, beta = _dev(gamma_h), _dev(beta_h)
    w, b = _dev(zq_inputs.weights(rng, H, H)), _dev(zq_inputs.bias(rng, H))
    wq, sw = zq.zq_quantize_weight_groupwise(w, g, 8)
    xq = torch.empty((M, H), dtype=torch.int8, device="cuda")
    st = torch.empty(M, dtype=torch.float32, device="cuda")
    out = torch.empty((M, H), dtype=torch.float16, device="cuda")

    def chain(_=0):
        zq.zq_layernorm_quant_tokenwise(x, gamma, beta, 1e-5, out=(xq, st))
        zq.zq_gemm_i8_dequant(xq, st, wq, sw, b, out=out)

    def fp16_chain(_=0):
        y = torch.nn.functional.layer_norm(x, (H,), gamma, beta, 1e-5)
        return torch.nn.functional.linear(y, w, b)

    graph_us = time_graph_median(graph_of(chain, 50), 50) * 1e3
    fp16_graph_us = time_graph_median(graph_of(fp16_chain, 50), 50) * 1e3
    eager = []
    for _ in range(5):
        for _ in range(10):
            chain()
        torch.cuda.synchronize()
        e0, e1 = _events(2)
        e0.record()
        for _ in range(50):
            chain()
        e1.record()
        torch.cuda.synchronize()
        eager.append(e0.elapsed_time(e1) * 1e3 / 50)
    return {"graph_us": graph_us, "eager_us": float(np.median(eager)), "fp16_graph_us": fp16_graph_us,
            "workload": "c1: LayerNorm+quant -> INT8 GeMM 768->768 at 128 tokens, 48 weight groups",
            "timing": "median of 5 repeats of 50 chains; eager = the same calls issued one by one through the "
                      "Python binding"}


def run_default(args):
    import paper_2206_01861_amd as zq
    zq.lib()
    torch.cuda.set_device(0)
    wl = FFCPair(zq)
    # exactly args.steps steps are timed: graphs of spg steps, spg the largest divisor of steps up to 10
    steps = max(1, args.steps)
    spg = max(d for d in range(1, 11) if steps % d == 0)
    replays = steps // spg
    g = graph_of(wl.step, spg)
    warm_replays = -(-max(0, args.warmup) // spg)
    for _ in range(warm_replays):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = _events(2)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / steps
    tops = wl.ops / (ms_per_step * 1e-3) / 1e12
    # the same chain as the median of five repeats of fifty steps, with the shader clock sampled meanwhile
    clk = {}
    step_median_ms = time_graph_median(graph_of(wl.step, 50), 50, repeats=5, clock=clk)
    sclk = clk.get("sclk_mhz")

    # per-call durations: each call replayed back to back in a graph of its own, on the same stream
    # (inputs and outputs of one call stay the same, so these are cache-warm figures)
    calls = {}
    for name, fn in (("layernorm_quant", wl.ln), ("gemm_ffc1", wl.gemm1), ("gelu_quant", wl.gelu),
                     ("gemm_ffc2", wl.gemm2)):
        calls[name] = time_graph_median(graph_of(fn, 50), 50, repeats=5, clock=clk) * 1e3          # us
        if name.startswith("gemm"):
            calls[name + "_sclk_mhz"] = clk.get("sclk_mhz")
    gemm_us = (calls["gemm_ffc1"] + calls["gemm_ffc2"]) / 2
    achieved = wl.gemm_ops / (gemm_us * 1e-6) / 1e12

    fused = None
    unfused = None
    if not args.no_fused:
        fused_ms = time_graph_median(graph_of(wl.fused_step, 50), 50)
        fused = {"ms_per_step": fused_ms, "TOPS": wl.ops / (fused_ms * 1e-3) / 1e12,
                 "gemm_ffc1_gelu_quant_us": time_graph_median(graph_of(wl.gemm1_gelu, 50), 50) * 1e3,
                 "gemm_ffc1_gelu_quant_with_fp16_output_us": time_graph_median(graph_of(wl.gemm1_gelu_keep, 50), 50) * 1e3,
                 "note": "zq_gemm_gelu_quant_tokenwise replaces GeMM 1 + GeLU+quant (three calls, the GeMM kernel "
                         "quantizes its own output rows); not the headline value"}
        torch.cuda.synchronize()
        expired = zq.quant_wait_expired(wl.ws)
        if expired:
            sys.exit("bench.py: %d waits of the in-kernel output quantization ran out; its figures are void" % expired)
        unfused_ms = time_graph_median(graph_of(wl.unfused_step, 20), 20)
        unfused = {"ms_per_step": unfused_ms, "fusion_speedup": unfused_ms / step_median_ms,
                   "note": "Fig. 2 (left): separate LayerNorm / GeLU (torch FP16), quantization, INT32 GeMM output and "
                           "dequantization kernels; eight launches instead of four"}

    fp16_ms = time_graph_median(graph_of(wl.fp16_step, 50), 50)
    fp16_gemm_us = time_graph_median(graph_of(lambda i: torch.nn.functional.linear(wl.x, wl.w1, wl.b1), 50), 50) * 1e3

    out = {
        "metric": "quantized-linear TOPS (W8A8, LayerNorm+quant -> GeMM -> GeLU+quant -> GeMM)",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": steps, "warmup": warm_replays * spg,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "c2: BERT-large FFC pair 1024->4096->1024, 4096 tokens (batch 32 x seq 128), "
                               "INT8 weights in 64 groups, token-wise INT8 activations",
                   "tokens": wl.M, "hidden": wl.H, "ffn": wl.F, "groups": wl.g,
                   "launch": "HIP graph replay, %d steps per graph" % spg,
                   "offline_weight_quant_ms": wl.weight_quant_ms},
        "ms_per_step_median": step_median_ms,
        "timing": "value: exactly `steps` steps between two events; every other figure: median of 5 repeats of "
                  ">= 50 launches (one graph replay per repeat)",
        "sclk_mhz": sclk if sclk is not None else "unavailable",
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": achieved / PEAK_INT8_TOPS, "traffic": GEMM_TRAFFIC_BYTES,
                     "traffic_source": GEMM_TRAFFIC_SOURCE + " (a constant from that profile, not measured in this run)",
                     "kernel": "gemm_tile_kernel (INT8 MFMA; one launch = one 4096-token GeMM of 2*4096*1024*4096 ops)",
                     "avg_launch_us": gemm_us},
        "calls_us": calls,
        "frontend_hbm": {
            "cache_warm": {
                "layernorm_quant_GBs": (3.0 * wl.M * wl.H + 4 * wl.H + 4 * wl.M) / (calls["layernorm_quant"] * 1e-6) / 1e9,
                "gelu_quant_GBs": (3.0 * wl.M * wl.F + 4 * wl.M) / (calls["gelu_quant"] * 1e-6) / 1e9,
                "note": "the same 12 MB / 48 MB every launch: served in part by the 256 MB Infinity Cache"},
            "rotated": rotated_frontends(zq, wl),
            "peak_GBs": PEAK_HBM_GBS},
        "fused_gelu_epilogue": fused,
        "unfused_pipeline": unfused,
        "fp16": {"ms_per_step": fp16_ms, "speedup_chain": fp16_ms / step_median_ms,
                 "gemm_ffc1_us": fp16_gemm_us, "speedup_gemm_ffc1": fp16_gemm_us / calls["gemm_ffc1"]},
        "paper_context": "ZeroQuant reports whole-model W8A8 speed-ups on A100-40GB only "
                         "(BERT-large seq128: 2.62x at batch 1 to 5.01x at batch 128); no kernel-level figures",
    }
    del g
    torch.cuda.empty_cache()
    ceil = measured_ceilings(zq)
    out["measured_ceilings"] = ceil
    out["roofline"]["frac_of_measured_mfma_ceiling"] = achieved / ceil["mfma_i8_TOPS_workload_codes"]
    out["roofline"]["frac_of_tile_traffic_ceiling"] = achieved / ceil["mfma_i8_TOPS_with_tile_traffic_workload_codes"]
    out["c1_chain_us"] = c1_chain(zq)
    if not args.no_rows:
        rows = []
        todo = ROWS
        if args.rows:
            todo = [(r.split(":")[0], int(r.split(":")[1]), "mfma" if int(r.split(":")[1]) > 128 else "hbm")
                    for r in args.rows.split(",")]
        for name, M, bound in todo:
            r = time_gemm(zq, name, M, comparators=not args.no_fp16_rows, oracle=not args.no_cpu)
            if bound == "mfma":
                r["roofline"] = {"bound": "mfma", "achieved": r["TOPS"], "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                                 "frac": r["frac_int8_peak"],
                                 "frac_of_measured_ceiling": r["TOPS"] / ceil["mfma_i8_TOPS_workload_codes"],
                                 "frac_of_tile_traffic_ceiling":
                                     r["TOPS"] / ceil["mfma_i8_TOPS_with_tile_traffic_workload_codes"]}
            else:
                floor_us = read_stream_floor_us(zq, r["bytes_min"])
                r["roofline"] = {"bound": "hbm", "achieved": r["GBs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                 "frac": r["frac_hbm_peak"],
                                 "frac_of_measured_ceiling": r["GBs"] / ceil["hbm_read_stream_GBs"],
                                 "read_stream_same_bytes_us": floor_us,
                                 "read_stream_same_bytes_note": "the read-only probe over the row's algorithmic bytes "
                                 "per launch, buffers rotating through 1.25 GB: what one launch needs to pull these "
                                 "bytes from HBM, without any arithmetic or output",
                                 "time_over_read_stream": r["us"] / floor_us}
            rows.append(r)
            torch.cuda.empty_cache()
        out["rows"] = rows
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


# ------------------------------------------------------------------ table ----
def _codes(gen, rows, cols, cfg):
    """INT8 activation codes with the value structure of the workload: N(0,1) rows with the
    configuration's outlier channels, quantized per row (torch ops; input preparation only)."""
    x = torch.randn((rows, cols), generator=gen, device="cuda")
    if cfg in ("c1", "c2"):
        n_out = 4 if cfg == "c1" else max(1, cols // 100)
        idx = torch.randperm(cols, generator=gen, device="cuda")[:n_out]
        x[:, idx] *= 20.0 if cfg == "c1" else 15.0
    elif cfg in ("c3", "c5"):
        x *= torch.exp(torch.empty((rows, 1), device="cuda").uniform_(np.log(0.5), np.log(2.0), generator=gen))
    else:
        n_ht = max(1, int(round(0.005 * cols)))
        idx = torch.randperm(cols, generator=gen, device="cuda")[:n_ht]
        t = torch.randn((rows, n_ht), generator=gen, device="cuda") / torch.sqrt(
            torch.clamp((torch.randn((rows, n_ht, 3), generator=gen, device="cuda") ** 2).mean(-1), min=1e-3))
        x[:, idx] = t
    a = x.abs().amax(dim=1, keepdim=True).clamp_min(1e-6)
    return torch.round(x * (127.0 / a)).clamp_(-127, 127).to(torch.int8), (a[:, 0] / 127.0).float()


def oracle_gemm_baseline(xq_t, st_t, codes_h, sw_t, bias_t, M):
    """The oracle's GeMM + epilogue on the host cores for one row of the table.  Prefill shapes (more
    than 64 tokens) are timed on the first 64 rows and the time is scaled by M / 64."""
    from oracle import zq_oracle as orc
    rows = min(M, 64)
    xq_h = xq_t[:rows].cpu().numpy()
    st_h, sw_h, b_h = st_t[:rows].cpu().numpy(), sw_t.cpu().numpy(), bias_t.cpu().numpy()
    t0 = time.perf_counter()
    acc = orc.matmul_i32(xq_h, codes_h)
    orc.dequant(acc, st_h, sw_h, b_h)
    dt = (time.perf_counter() - t0) * (M / rows)
    N, K = codes_h.shape
    return {"value": 2.0 * M * N * K / dt / 1e12, "unit": "TOPS", "seconds": dt, "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": ("all %d rows" % M) if rows == M else ("first 64 rows, time scaled by %d/64" % M)}


def read_stream_floor_us(zq, nbytes, min_launches=50):
    """What the read-only probe (include/zq_probe.h) takes for `nbytes` per launch, the launches walking
    through a 1.25 GB buffer: the time a single launch needs just to pull that many bytes out of HBM,
    launch and ramp included.  The decode rows are read against it."""
    n = max(4096, int(nbytes) // 4096 * 4096)
    big = torch.empty(1280 << 20, dtype=torch.uint8, device="cuda").random_(0, 256)
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    nset = max(1, big.numel() // n)
    reps = -(-min_launches // nset) * nset
    g = graph_of(lambda i: zq.zq_probe_read_stream(big[(i % nset) * n:(i % nset) * n + n], sink), reps)
    ms = time_graph_median(g, reps)
    del g, big
    torch.cuda.empty_cache()
    return ms * 1e3


def time_gemm(zq, name, M, min_launches=50, repeats=5, comparators=True, oracle=False):
    """One GeMM of the workload table: median of `repeats` timed graph replays of at least
    `min_launches` launches each.  Up to 64 tokens the operands rotate through more than 512 MB."""
    K, N, g, bits = zq_inputs.LINEARS[name]
    cfg = name.split("_")[0]
    gen = torch.Generator(device="cuda").manual_seed(zq_inputs.BASE_SEED % (2 ** 31) + M)
    wbytes = N * K * bits // 8
    per_set = wbytes + M * K + 2 * M * N
    nset = int(max(1, min(32, -(-ROTATE_BYTES // per_set)))) if M <= 64 else 1
    sets = []
    for _ in range(nset):
        xq, st = _codes(gen, M, K, cfg)
        w = (torch.randn((N, K), generator=gen, device="cuda") * 0.02 *
             torch.exp(torch.empty((N, 1), device="cuda").uniform_(np.log(0.3), np.log(3.0), generator=gen))).half()
        wq, sw = zq.zq_quantize_weight_groupwise(w, g, bits)
        del w
        out = torch.empty((M, N), dtype=torch.float16, device="cuda")
        sets.append((xq, st, wq, sw, out))
    bias = (torch.randn(N, generator=gen, device="cuda") * 0.01).half()
    nws = zq.gemm_workspace_bytes(M, N, K, bits)
    ws = zq.new_workspace(nws)
    fn = zq.zq_gemm_i8_dequant if bits == 8 else zq.zq_gemm_w4a8_dequant

    def run(i):
        xq, st, wq, sw, out = sets[i % nset]
        fn(xq, st, wq, sw, bias, workspace=ws, out=out)

    # launches per graph: a whole number of passes over the rotating sets; long launches need fewer
    # for a stable figure (a 16384-token GeMM is milliseconds), the floor stays at min_launches / 5
    ops = 2.0 * M * N * K
    reps = -(-min_launches // nset) * nset
    if ops > 1e12:
        reps = max(10, min_launches // 5)
    gq = graph_of(run, reps)
    clk = {}
    best = time_graph_median(gq, reps, repeats=repeats, warm=1, clock=clk)          # ms per call
    clock = clk.get("sclk_mhz")
    del gq
    fbest = lib_int8 = None
    if comparators:
        xf = torch.randn((M, K), device="cuda", dtype=torch.float16)
        wfs = [torch.randn((N, K), device="cuda", dtype=torch.float16) * 0.02
               for _ in range(min(nset, max(1, ROTATE_BYTES // (2 * N * K) + 1)) if M <= 64 else 1)]
        freps = reps if M <= 64 else 10
        gf = graph_of(lambda i: torch.nn.functional.linear(xf, wfs[i % len(wfs)], bias), freps)
        fbest = time_graph_median(gf, freps, repeats=3, warm=1)
        del xf, wfs, gf
        # The vendor library's own INT8 GeMM (torch._int_mm -> hipBLASLt: INT32 output, no scales, no
        # bias) on the prefill shapes, as a second comparator.
        if M > 128:
            try:
                xi = torch.randint(-127, 128, (M, K), device="cuda", dtype=torch.int8)
                wi = torch.randint(-127, 128, (N, K), device="cuda", dtype=torch.int8).t()
                torch._int_mm(xi, wi)
                gi = graph_of(lambda i: torch._int_mm(xi, wi), 5)
                lib_int8 = time_graph_median(gi, 5, repeats=3, warm=1)
                del xi, wi, gi
            except Exception:                       # not every build routes _int_mm to a library kernel
                lib_int8 = None
    bytes_min = M * K + wbytes + 4 * M + 4 * g + 2 * N + 2 * M * N
    variant = zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, bits, nws))
    row = {"linear": name, "M": M, "N": N, "K": K, "w_bits": bits, "groups": g, "schedule": variant,
           "us": best * 1e3, "TOPS": ops / (best * 1e-3) / 1e12, "GBs": bytes_min / (best * 1e-3) / 1e9,
           "frac_int8_peak": ops / (best * 1e-3) / 1e12 / PEAK_INT8_TOPS,
           "frac_hbm_peak": bytes_min / (best * 1e-3) / 1e9 / PEAK_HBM_GBS,
           "ops": ops, "bytes_min": bytes_min,
           "timing": "median of %d repeats of %d launches (one graph replay each)" % (repeats, reps),
           "rotating_sets": nset, "rotating_bytes": nset * per_set,
           "sclk_mhz": clock if clock is not None else "unavailable",
           "fp16_us": None if fbest is None else fbest * 1e3,
           "speedup_vs_fp16": None if fbest is None else fbest / best,
           "lib_int8_us": None if lib_int8 is None else lib_int8 * 1e3,
           "speedup_vs_lib_int8": None if lib_int8 is None else lib_int8 / best}
    if oracle:
        xq, st, wq, sw, _ = sets[0]
        if bits == 8:
            codes_h = wq.cpu().numpy()
        else:
            from oracle import zq_oracle as orc
            codes_h = orc.unpack_int4(wq.cpu().numpy())
        row["cpu_baseline"] = oracle_gemm_baseline(xq, st, codes_h, sw, bias, M)
    return row


def time_gemm_a16(zq, name, M, reps_target=40):
    """W8A16 (FP16 activations x INT8 weights) on a QKV linear: the setting the paper uses for the input
    of the QKV GeMM of its largest model (Sec. 5)."""
    K, N, g, bits = zq_inputs.LINEARS[name]
    gen = torch.Generator(device="cuda").manual_seed(zq_inputs.BASE_SEED % (2 ** 31) + 7 * M)
    wbytes = N * K
    nset = int(max(1, min(32, -(-(640 << 20) // wbytes)))) if M <= 128 else 1
    x = (torch.randn((M, K), generator=gen, device="cuda") *
         torch.exp(torch.empty((M, 1), device="cuda").uniform_(np.log(0.5), np.log(2.0), generator=gen))).half()
    sets = []
    for _ in range(nset):
        w = (torch.randn((N, K), generator=gen, device="cuda") * 0.02).half()
        wq, sw = zq.zq_quantize_weight_groupwise(w, g, 8)
        del w
        sets.append((wq, sw))
    bias = (torch.randn(N, generator=gen, device="cuda") * 0.01).half()
    out = torch.empty((M, N), dtype=torch.float16, device="cuda")
    nws = zq.gemm_w8a16_workspace_bytes(M, N, K)
    ws = zq.new_workspace(nws)

    def run(i):
        wq, sw = sets[i % nset]
        zq.zq_gemm_w8a16_dequant(x, wq, sw, bias, workspace=ws, out=out)

    reps = max(nset, reps_target // max(1, nset) * nset) if M <= 64 else 10
    gq = graph_of(run, reps)
    best = min(time_graph(gq, 3, reps, warm=1) for _ in range(3))
    wfs = [torch.randn((N, K), device="cuda", dtype=torch.float16) * 0.02
           for _ in range(min(nset, max(1, (640 << 20) // (2 * N * K) + 1)) if M <= 64 else 1)]
    gf = graph_of(lambda i: torch.nn.functional.linear(x, wfs[i % len(wfs)], bias), reps)
    fbest = min(time_graph(gf, 3, reps, warm=1) for _ in range(2))
    del wfs, gf, gq
    ops = 2.0 * M * N * K
    bytes_min = 2 * M * K + wbytes + 4 * g + 2 * N + 2 * M * N
    return {"linear": name + "/w8a16", "M": M, "N": N, "K": K, "w_bits": 8, "groups": g,
            "schedule": "stream_a16" if (M <= 64 and K % 256 == 0) else ("tile_a16" if K % 64 == 0 else "simple_a16"),
            "us": best * 1e3, "TOPS": ops / (best * 1e-3) / 1e12, "GBs": bytes_min / (best * 1e-3) / 1e9,
            "frac_int8_peak": None, "frac_fp16_peak": ops / (best * 1e-3) / 1e12 / 2500.0,
            "frac_hbm_peak": bytes_min / (best * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "fp16_us": fbest * 1e3, "speedup_vs_fp16": fbest / best, "rotating_sets": nset}


def run_table(args):
    import paper_2206_01861_amd as zq
    zq.lib()
    rows = []
    cases = []
    for name in zq_inputs.LINEARS:
        cfg = name.split("_")[0]
        for M in zq_inputs.TOKENS[cfg]:
            cases.append((name, M))
    if args.only:
        cases = [c for c in cases if c[0].startswith(args.only)]
    for name, M in cases:
        r = time_gemm(zq, name, M)
        rows.append(r)
        lib = "" if r["lib_int8_us"] is None else "  lib int8 %8.1f us x%.2f" % (r["lib_int8_us"], r["speedup_vs_lib_int8"])
        print("%-8s M=%-6d %-14s %9.1f us %8.1f TOPS %8.1f GB/s  int8 %.3f hbm %.3f  fp16 %8.1f us x%.2f%s" % (
            name, M, r["schedule"], r["us"], r["TOPS"], r["GBs"], r["frac_int8_peak"], r["frac_hbm_peak"],
            r["fp16_us"], r["speedup_vs_fp16"], lib), file=sys.stderr, flush=True)
        torch.cuda.empty_cache()
    # W8A16 on the QKV linears (the GeMM whose input the paper keeps in FP16 for its largest model)
    for name, M in cases:
        if not name.endswith("_qkv"):
            continue
        r = time_gemm_a16(zq, name, M)
        rows.append(r)
        print("%-14s M=%-4d %-11s %9.1f us %8.1f TFLOPS %8.1f GB/s  hbm %.3f  fp16 %8.1f us x%.2f" % (
            r["linear"], M, r["schedule"], r["us"], r["TOPS"], r["GBs"], r["frac_hbm_peak"], r["fp16_us"],
            r["speedup_vs_fp16"]), file=sys.stderr, flush=True)
        torch.cuda.empty_cache()
    path = os.path.abspath(args.table_json)
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        json.dump(rows, f, indent=1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--rows", default="", help="comma-separated linear:tokens pairs replacing the default rows")
    ap.add_argument("--table", action="store_true", help="time every workload shape")
    ap.add_argument("--table-json", default=os.path.join(ROOT, "bench_table.json"),
                    help="with --table: where the rows are written as JSON")
    ap.add_argument("--only", default="", help="with --table: restrict to linears whose name starts with this")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-rows", action="store_true", help="skip the per-GeMM rows (large prefill and rotated decode shapes)")
    ap.add_argument("--no-fp16-rows", action="store_true", help="rows without their FP16 comparator")
    ap.add_argument("--no-fused", action="store_true",
                    help="skip the extra three-call chain (keeps a profile of the default run to the headline kernels)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device copy, the known-size kernel that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the quantized linear layer has no cross-GPU step "
                 "(run with --gpus 1)")
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.table:
        run_table(args)
    else:
        run_default(args)


if __name__ == "__main__":
    main()
