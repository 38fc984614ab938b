"""Shape autotuner for the GeMM calls of libzq.

The paper ranks its GeMM schedules by measuring them offline and picks one at run time from
batch x sequence length (App. D).  This module does the same on the installed GPU: for a GeMM
shape it times every schedule the library supports (and, for the weight-streaming schedules, the
cost model's cut of the matrix and its neighbours) under HIP-graph replay, with the weight buffers
rotated through more than the Infinity Cache holds when the token count is small, and registers
the fastest with zq_tune_set.  Results can be saved to and loaded from a JSON file.

    python -m paper_2206_01861_amd.autotune --shape 64,24576,6144,8 --shape 16,4096,16384,4 --save tuned.json
"""
import argparse
import json

import torch

from . import binding as zq

SKINNY, SKINNY_SPLITK = 3, 4
ROTATE_BYTES = 640 << 20          # decode shapes: weights rotate through more than the 256 MB cache


def _time_us(fn, nsets, reps=3):
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        for i in range(min(2, nsets)):
            fn(i)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        calls = max(nsets, 8)
        with torch.cuda.graph(g, stream=s):
            for i in range(calls):
                fn(i % nsets)
        g.replay()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e3 / (2 * calls))
    return best


def _cuts(M, N, K, bits):
    """The cost model's cut and its neighbours: one consumer more or fewer, half or double the K split."""
    strips, stages = N // 16, K // 256
    ws = zq.gemm_workspace_bytes(M, N, K, bits)
    rb0, ks0, c0 = zq.gemm_stream_plan(M, N, K, bits, ws)
    cuts = {(rb0, ks0)}
    for c in (c0 - 1, c0 + 1, c0 + 2):
        if 1 <= c <= 8:
            for rb in {-(-strips // c), min(strips, 256 * max(1, round(strips / (256.0 * c))))}:
                if 1 <= rb <= strips and -(-strips // rb) <= 8:
                    for ks in {ks0, max(1, ks0 // 2), min(stages, ks0 * 2)}:
                        cuts.add((rb, ks))
    if ks0 > 1:
        cuts.add((min(strips, 256), 1))
    return sorted(c for c in cuts if 1 <= c[1] <= stages)


def tune_shape(M, N, K, bits, m_lo=None, m_hi=None, verbose=False):
    """Time every candidate for one shape, register the best, return (best_entry, all_results)."""
    dev = "cuda"
    gen = torch.Generator(device=dev).manual_seed(1234)
    wbytes = N * K * bits // 8
    nsets = 1 if M > 128 else int(max(2, min(32, -(-ROTATE_BYTES // wbytes))))
    xq = torch.randint(-127, 128, (M, K), generator=gen, device=dev, dtype=torch.int8)
    ws_ = [torch.randint(0, 256, (N, K * bits // 8), generator=gen, device=dev, dtype=torch.uint8) for _ in range(nsets)]
    if bits == 8:
        ws_ = [w.view(torch.int8) for w in ws_]
    groups = max(1, N // 64) if N % 64 == 0 else N // 16
    st = torch.rand(M, generator=gen, device=dev) * 0.1 + 0.01
    sw = torch.rand(groups, generator=gen, device=dev) * 1e-3 + 1e-4
    bias = (torch.randn(N, generator=gen, device=dev) * 0.01).half()
    out = torch.empty((M, N), dtype=torch.float16, device=dev)
    fn = zq.zq_gemm_i8_dequant if bits == 8 else zq.zq_gemm_w4a8_dequant
    m_lo = M if m_lo is None else m_lo
    m_hi = M if m_hi is None else m_hi

    candidates = []
    v_count = 0
    while zq.gemm_variant_name(v_count) is not None:
        v_count += 1
    for v in range(v_count):
        if v in (SKINNY, SKINNY_SPLITK):
            continue
        if zq.gemm_variant_name(v) == "simple" and M * N * K > (1 << 31):
            continue                                  # the fallback schedule is never competitive at size
        candidates.append((v, 0, 0))
    if M <= 128 and K % 256 == 0:
        for rb, ks in _cuts(M, N, K, bits):
            candidates.append((SKINNY if ks == 1 else SKINNY_SPLITK, rb, ks))

    results = []
    before = zq.tune_count()
    for v, rb, ks in candidates:
        try:
            zq.tune_set(m_lo, m_hi, N, K, bits, v, rb, ks)
        except zq.ZQError:
            continue
        nws = zq.gemm_workspace_bytes(M, N, K, bits)
        wsb = zq.new_workspace(nws)
        if zq.gemm_choose_variant(M, N, K, bits, nws) != v:
            continue                                  # not runnable for this shape
        us = _time_us(lambda i: fn(xq, st, ws_[i], sw, bias, workspace=wsb, out=out), nsets)
        results.append({"variant": v, "name": zq.gemm_variant_name(v), "row_blocks": rb, "k_splits": ks, "us": us})
        if verbose:
            print("  %-14s rb=%-5d ks=%-3d %8.1f us" % (zq.gemm_variant_name(v), rb, ks, us), flush=True)
    assert zq.tune_count() >= before
    best = min(results, key=lambda r: r["us"])
    zq.tune_set(m_lo, m_hi, N, K, bits, best["variant"], best["row_blocks"], best["k_splits"])
    entry = {"m_lo": m_lo, "m_hi": m_hi, "N": N, "K": K, "w_bits": bits, "variant": best["variant"],
             "row_blocks": best["row_blocks"], "k_splits": best["k_splits"], "us": best["us"]}
    return entry, results


def load(path):
    """Register every entry of a file written by save()."""
    with open(path) as f:
        entries = json.load(f)
    for e in entries:
        zq.tune_set(e["m_lo"], e["m_hi"], e["N"], e["K"], e["w_bits"], e["variant"], e["row_blocks"], e["k_splits"])
    return len(entries)


def save(entries, path):
    with open(path, "w") as f:
        json.dump(entries, f, indent=1)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--shape", action="append", default=[], help="M,N,K,w_bits (repeatable)")
    ap.add_argument("--save", default="", help="write the winning entries to this JSON file")
    args = ap.parse_args()
    zq.lib()
    entries = []
    for sh in args.shape:
        M, N, K, bits = (int(v) for v in sh.split(","))
        default_us = None
        print("shape M=%d N=%d K=%d bits=%d" % (M, N, K, bits), flush=True)
        entry, results = tune_shape(M, N, K, bits, verbose=True)
        entries.append(entry)
        print("  -> %s rb=%d ks=%d %.1f us" % (zq.gemm_variant_name(entry["variant"]), entry["row_blocks"],
                                               entry["k_splits"], entry["us"]), flush=True)
    if args.save:
        save(entries, args.save)


if __name__ == "__main__":
    main()
