#!/usr/bin/env python3
"""Benchmark of the quantized linear layer on one MI355X.

Default run (`python bench.py`): the BERT-large feed-forward pair of the
paper's BERT-large workload (batch 32 x sequence 128 = 4096 tokens),
  LayerNorm+quant -> INT8 GeMM 1024->4096 (+bias) -> GeLU+quant -> INT8 GeMM 4096->1024 (+bias),
with inputs resident in HBM.  A step is one pass of that chain.  Prints ONE JSON
line: whole-chain throughput in TOPS, the roofline of the dominant kernel (the
tiled INT8 GeMM, launched twice per step), the same chain in FP16 through
torch (hipBLASLt / rocBLAS) as the speed-up comparator, and the CPU oracle
timed on the host cores.

`python bench.py --table` additionally times every linear of every workload
shape (prefill: TOPS vs the INT8 matrix-core peak; decode: GB/s vs HBM, with
buffers rotated through more than 512 MB so the Infinity Cache cannot serve
them) and writes gpurun_out/bench_table.json; it prints nothing else.
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
PEAK_FP16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


def _events(n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class FFCPair:
    """Workload c2: tensors resident on the GPU, weights quantized once (offline step)."""

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
        t0 = torch.cuda.Event(enable_timing=True)
        t1 = torch.cuda.Event(enable_timing=True)
        zq.zq_quantize_weight_groupwise(self.w1, groups, 8)      # warm
        torch.cuda.synchronize()
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
        self.ops = 2.0 * tokens * (hidden * ffn + ffn * hidden)
        self.gemm_ops = 2.0 * tokens * hidden * ffn          # per GeMM launch (both are equal)

    def step(self, ev=None):
        zq = self.zq
        if ev is not None:
            ev[0].record()
        zq.zq_layernorm_quant_tokenwise(self.x, self.gamma, self.beta, 1e-5, out=(self.xq, self.st))
        if ev is not None:
            ev[1].record()
        zq.zq_gemm_i8_dequant(self.xq, self.st, self.wq1, self.sw1, self.b1, out=self.h)
        if ev is not None:
            ev[2].record()
        zq.zq_gelu_quant_tokenwise(self.h, None, out=(self.hq, self.st2))
        if ev is not None:
            ev[3].record()
        zq.zq_gemm_i8_dequant(self.hq, self.st2, self.wq2, self.sw2, self.b2, out=self.o)
        if ev is not None:
            ev[4].record()

    def fp16_step(self):
        F = torch.nn.functional
        y = F.layer_norm(self.x, (self.H,), self.gamma, self.beta, 1e-5)
        h = F.linear(y, self.w1, self.b1)
        a = F.gelu(h)
        return F.linear(a, self.w2, self.b2)


def time_loop(fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = _events(2)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    return max(e0.elapsed_time(e1), 0.0), wall


def cpu_baseline(wl, budget_tokens=1024):
    """The oracle, as it stands, on the host cores, over the first `budget_tokens` tokens of the same chain."""
    from oracle import zq_oracle as orc
    m = min(budget_tokens, wl.M)
    x = wl.x_h[:m]
    wq1, sw1, _ = orc.quantize_weight_groupwise(wl.w1_h, wl.g, 8)
    wq2, sw2, _ = orc.quantize_weight_groupwise(wl.w2_h, wl.g, 8)
    t0 = time.perf_counter()
    _, y32 = orc.layernorm(x, wl.gamma_h, wl.beta_h, 1e-5)
    xq, st = orc.quant_tokenwise(y32)
    acc = orc.matmul_i32(xq, wq1)
    ref, _ = orc.dequant(acc, st, sw1, wl.b1_h)
    h16 = ref.astype(np.float16)
    _, g32 = orc.gelu(h16, None)
    hq, st2 = orc.quant_tokenwise(g32)
    acc2 = orc.matmul_i32(hq, wq2)
    orc.dequant(acc2, st2, sw2, wl.b2_h)
    dt = time.perf_counter() - t0
    ops = 2.0 * m * (wl.H * wl.F * 2)
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "first %d of %d tokens of the same chain, %.1f s wall" % (m, wl.M, dt)}


def run_default(args):
    import paper_2206_01861_amd as zq
    zq.lib()
    torch.cuda.set_device(0)
    wl = FFCPair(zq)
    # whole-chain throughput
    ms, wall_ms = time_loop(wl.step, args.steps, args.warmup)
    ms_per_step = ms / args.steps
    tops = wl.ops / (ms_per_step * 1e-3) / 1e12
    # per-call breakdown, events on the same stream inside a second timed region
    n_prof = min(args.steps, 200)
    evs = [_events(5) for _ in range(n_prof)]
    for i in range(n_prof):
        wl.step(evs[i])
    torch.cuda.synchronize()
    per = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(4)] for e in evs])     # ms
    call_ms = per.mean(axis=0)
    gemm_ms = float((call_ms[1] + call_ms[3]) / 2)
    achieved = wl.gemm_ops / (gemm_ms * 1e-3) / 1e12
    # FP16 comparator: the same chain through torch
    fms, _ = time_loop(wl.fp16_step, args.steps, args.warmup)
    fp16_ms = fms / args.steps
    fe = [_events(2) for _ in range(50)]
    for a, b in fe:
        a.record()
        torch.nn.functional.linear(wl.h, wl.w2, wl.b2)
        b.record()
    torch.cuda.synchronize()
    fp16_gemm_ms = float(np.mean([a.elapsed_time(b) for a, b in fe]))
    out = {
        "metric": "quantized-linear TOPS (W8A8, LayerNorm+quant -> GeMM -> GeLU+quant -> GeMM)",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "c2: BERT-large FFC pair 1024->4096->1024, 4096 tokens (batch 32 x seq 128), "
                               "INT8 weights in 64 groups, token-wise INT8 activations",
                   "tokens": wl.M, "hidden": wl.H, "ffn": wl.F, "groups": wl.g,
                   "offline_weight_quant_ms": wl.weight_quant_ms},
        "roofline": {"bound": "mfma", "kernel": "gemm_tile_kernel (INT8 MFMA, one launch = one 4096x4096x1024 GeMM)",
                     "achieved": achieved, "peak": PEAK_INT8_TOPS / 1e3 * 1e3, "unit": "TOP/s",
                     "frac": achieved / PEAK_INT8_TOPS, "traffic": None,
                     "avg_launch_us": gemm_ms * 1e3},
        "calls_us": {"layernorm_quant": call_ms[0] * 1e3, "gemm_ffc1": call_ms[1] * 1e3,
                     "gelu_quant": call_ms[2] * 1e3, "gemm_ffc2": call_ms[3] * 1e3},
        "frontend_hbm": {
            "layernorm_quant_GBs": (3.0 * wl.M * wl.H + 4 * wl.H + 4 * wl.M) / (call_ms[0] * 1e-3) / 1e9,
            "gelu_quant_GBs": (3.0 * wl.M * wl.F + 4 * wl.M) / (call_ms[2] * 1e-3) / 1e9,
            "peak_GBs": PEAK_HBM_GBS},
        "fp16": {"ms_per_step": fp16_ms, "speedup_chain": fp16_ms / ms_per_step,
                 "gemm_ffc2_us": fp16_gemm_ms * 1e3, "speedup_gemm_ffc2": fp16_gemm_ms / (call_ms[3])},
        "paper_context": "ZeroQuant reports whole-model W8A8 speed-ups on A100-40GB only "
                         "(BERT-large seq128: 2.62x at batch 1 to 5.01x at batch 128); no kernel-level figures",
    }
    out["roofline"]["peak"] = PEAK_INT8_TOPS
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


# ------------------------------------------------------------------ table ----
def _rot_count(bytes_per_set, target=640 << 20, cap=64):
    return int(max(1, min(cap, -(-target // max(bytes_per_set, 1)))))


def time_gemm(zq, name, M, reps=50):
    K, N, g, bits = zq_inputs.LINEARS[name]
    qmax = 127 if bits == 8 else 7
    gen = torch.Generator(device="cuda").manual_seed(1 + M)
    wbytes = N * K * bits // 8
    nset = _rot_count(wbytes + M * K + 2 * M * N) if M <= 64 else 1
    sets = []
    for _ in range(nset):
        xq = torch.randint(-127, 128, (M, K), generator=gen, device="cuda", dtype=torch.int8)
        if bits == 8:
            wq = torch.randint(-qmax, qmax + 1, (N, K), generator=gen, device="cuda", dtype=torch.int8)
        else:
            wq = torch.randint(0, 256, (N, K // 2), generator=gen, device="cuda", dtype=torch.uint8)
        out = torch.empty((M, N), dtype=torch.float16, device="cuda")
        sets.append((xq, wq, out))
    st = torch.rand(M, device="cuda") * 0.1 + 0.01
    sw = torch.rand(g, device="cuda") * 1e-3 + 1e-4
    bias = (torch.randn(N, device="cuda") * 0.01).half()
    nws = zq.gemm_workspace_bytes(M, N, K, bits)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    fn = zq.zq_gemm_i8_dequant if bits == 8 else zq.zq_gemm_w4a8_dequant

    def run(i):
        xq, wq, out = sets[i % nset]
        fn(xq, st, wq, sw, bias, workspace=ws, out=out)

    for i in range(max(5, nset)):
        run(i)
    torch.cuda.synchronize()
    best = None
    for _ in range(5):
        e0, e1 = _events(2)
        e0.record()
        for i in range(reps):
            run(i)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) / reps
        best = t if best is None else min(best, t)
    # FP16 comparator on the same shape (one buffer set is enough: it is a comparator)
    xf = torch.randn((M, K), device="cuda", dtype=torch.float16)
    wf = torch.randn((N, K), device="cuda", dtype=torch.float16) * 0.02
    for _ in range(5):
        torch.nn.functional.linear(xf, wf, bias)
    torch.cuda.synchronize()
    fbest = None
    for _ in range(3):
        e0, e1 = _events(2)
        e0.record()
        for i in range(reps):
            torch.nn.functional.linear(xf, wf, bias)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) / reps
        fbest = t if fbest is None else min(fbest, t)
    del xf, wf
    ops = 2.0 * M * N * K
    bytes_min = M * K + wbytes + 4 * M + 4 * g + 2 * N + 2 * M * N
    variant = zq.gemm_variant_name(zq.gemm_choose_variant(M, N, K, bits, nws))
    return {"linear": name, "M": M, "N": N, "K": K, "w_bits": bits, "groups": g, "schedule": variant,
            "us": best * 1e3, "TOPS": ops / (best * 1e-3) / 1e12, "GBs": bytes_min / (best * 1e-3) / 1e9,
            "frac_int8_peak": ops / (best * 1e-3) / 1e12 / PEAK_INT8_TOPS,
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
        print("%-8s M=%-6d %-14s %9.1f us %8.1f TOPS %8.1f GB/s  int8 %.3f hbm %.3f  fp16 x%.2f" % (
            name, M, r["schedule"], r["us"], r["TOPS"], r["GBs"], r["frac_int8_peak"], r["frac_hbm_peak"],
            r["speedup_vs_fp16"]), file=sys.stderr, flush=True)
        torch.cuda.empty_cache()
    os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
    with open(os.path.join(ROOT, "gpurun_out", "bench_table.json"), "w") as f:
        json.dump(rows, f, indent=1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--table", action="store_true", help="time every workload shape; writes gpurun_out/bench_table.json")
    ap.add_argument("--only", default="", help="with --table: restrict to linears whose name starts with this")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
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
