#!/usr/bin/env python3
"""Writes tests/golden/quantizer_small.txt: the oracle's codes and scales for a small seeded case.

The paper prints no worked numeric example of its quantizer (App. A.2), so this file is not a
paper value; it freezes what oracle/ computes today, so that an unnoticed change to the oracle's
arithmetic shows up as a diff.  Calls only oracle/ and the seeded input generator.
Run from the repository root:  python tests/golden/make_quantizer_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import zq_inputs  # noqa: E402
from oracle import zq_oracle as orc  # noqa: E402


def case():
    rng = zq_inputs.rng_for(0, 42)
    w = zq_inputs.weights(rng, 32, 32)                     # fp16 [32,32], 2 groups of 16 rows
    x = zq_inputs.activations(rng, 4, 32, outlier_frac=0.05, outlier_scale=8.0)
    return w, x


def lines():
    w, x = case()
    out = ["# quantizer_small: seeded fp16 inputs (hex), oracle outputs.  See make_quantizer_golden.py",
           "w_fp16_hex " + w.view(np.uint16).tobytes().hex(),
           "x_fp16_hex " + x.view(np.uint16).tobytes().hex()]
    for bits in (8, 4):
        wq, s_w, codes = orc.quantize_weight_groupwise(w, 2, bits)
        out.append("w%d_packed_hex %s" % (bits, np.ascontiguousarray(wq).view(np.uint8).tobytes().hex()))
        out.append("w%d_scale_hex %s" % (bits, s_w.view(np.uint32).tobytes().hex()))
    xq, s_tok = orc.quant_tokenwise(x.astype(np.float32))
    out.append("x_codes_hex " + xq.view(np.uint8).tobytes().hex())
    out.append("x_scale_hex " + s_tok.view(np.uint32).tobytes().hex())
    acc = orc.matmul_i32(xq, orc.quantize_weight_groupwise(w, 2, 8)[2])
    out.append("acc_i32 " + " ".join(str(int(v)) for v in acc.ravel()))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "quantizer_small.txt")
    with open(path, "w") as f:
        f.write("\n".join(lines()) + "\n")
    print("wrote", path)
