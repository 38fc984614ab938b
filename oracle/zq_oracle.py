"""ctypes front for the plain-C CPU oracle (oracle/zq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  Nothing here touches the GPU library, and
the GPU library never imports this package.

Every function takes and returns numpy arrays; fp16 tensors travel as
numpy.float16 arrays (their bit patterns are handed to C as uint16).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zq_oracle.c")
_LIB = os.path.join(_HERE, "libzq_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP, no contraction)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-std=c99", "-Wall", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.zq_oracle_quantize_block.restype = ctypes.c_float
        _lib.zq_oracle_quantize_weight_groupwise.restype = ctypes.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def num_threads():
    """Threads the OpenMP loops use (OMP_NUM_THREADS or the core count)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return int(v.split(",")[0])
        except ValueError:
            pass
    return os.cpu_count() or 1


def half_to_float(h):
    h = _c(h, np.float16)
    out = np.empty(h.shape, np.float32)
    _load().zq_oracle_half_to_float(_p(h), ctypes.c_long(h.size), _p(out))
    return out


def quantize_block(v, qmax):
    """App. A.2 quantizer over one block sharing a scale -> (codes int8, scale fp32)."""
    v = _c(v, np.float32)
    q = np.empty(v.shape, np.int8)
    s = _load().zq_oracle_quantize_block(_p(v), ctypes.c_long(v.size), ctypes.c_int(qmax), _p(q))
    return q, np.float32(s)


def quant_tokenwise(y32):
    """Sec. 4.1 token-wise INT8: y32 fp32 [M,K] -> (xq int8 [M,K], s_tok fp32 [M])."""
    y32 = _c(y32, np.float32)
    M, K = y32.shape
    xq = np.empty((M, K), np.int8)
    s = np.empty(M, np.float32)
    _load().zq_oracle_quant_tokenwise(_p(y32), ctypes.c_long(M), ctypes.c_long(K), _p(xq), _p(s))
    return xq, s


def quantize_weight_groupwise(w16, groups, bits):
    """Sec. 4.1 group-wise weights: w fp16 [N,K] -> (wq, s_w fp32 [g], codes int8 [N,K]).

    wq is int8 [N,K] for bits=8 and packed uint8 [N,K/2] for bits=4.
    """
    w16 = _c(w16, np.float16)
    N, K = w16.shape
    wq = np.empty((N, K), np.int8) if bits == 8 else np.empty((N, K // 2), np.uint8)
    s_w = np.empty(groups, np.float32)
    codes = np.empty((N, K), np.int8)
    rc = _load().zq_oracle_quantize_weight_groupwise(
        _p(w16), ctypes.c_long(N), ctypes.c_long(K), ctypes.c_long(groups),
        ctypes.c_int(bits), _p(wq), _p(s_w), _p(codes))
    if rc != 0:
        raise ValueError("bad arguments to quantize_weight_groupwise")
    return wq, s_w, codes


def unpack_int4(packed):
    packed = _c(packed, np.uint8)
    codes = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), np.int8)
    _load().zq_oracle_unpack_int4(_p(packed), ctypes.c_long(packed.size), _p(codes))
    return codes


def layernorm(x16, gamma16, beta16, eps):
    """fp64 LayerNorm over the last axis -> (y64, y32)."""
    x16 = _c(x16, np.float16)
    gamma16 = _c(gamma16, np.float16)
    M, K = x16.shape
    y64 = np.empty((M, K), np.float64)
    y32 = np.empty((M, K), np.float32)
    b = _p(_c(beta16, np.float16)) if beta16 is not None else None
    _load().zq_oracle_layernorm(_p(x16), _p(gamma16), b, ctypes.c_double(eps),
                                ctypes.c_long(M), ctypes.c_long(K), _p(y64), _p(y32))
    return y64, y32


def gelu(h16, bias16, approx_tanh=False):
    """fp64 bias-add + GeLU -> (y64, y32)."""
    h16 = _c(h16, np.float16)
    M, N = h16.shape
    y64 = np.empty((M, N), np.float64)
    y32 = np.empty((M, N), np.float32)
    b = _p(_c(bias16, np.float16)) if bias16 is not None else None
    _load().zq_oracle_gelu(_p(h16), b, ctypes.c_int(1 if approx_tanh else 0),
                           ctypes.c_long(M), ctypes.c_long(N), _p(y64), _p(y32))
    return y64, y32


def gelu_f64(u64, approx_tanh=False):
    """GeLU of fp64 values (any shape) -> fp64."""
    u64 = _c(u64, np.float64)
    y = np.empty_like(u64)
    _load().zq_oracle_gelu_f64(_p(u64), ctypes.c_int(1 if approx_tanh else 0), ctypes.c_long(u64.size), _p(y))
    return y


def matmul_i32(xq, wq):
    """acc[m,n] = sum_k xq[m,k]*wq[n,k] in int32."""
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    _load().zq_oracle_matmul_i32(_p(xq), _p(wq), ctypes.c_long(M), ctypes.c_long(N),
                                 ctypes.c_long(K), _p(acc))
    return acc


def matmul_i64(xq, wq):
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    acc = np.empty((M, N), np.int64)
    _load().zq_oracle_matmul_i64(_p(xq), _p(wq), ctypes.c_long(M), ctypes.c_long(N),
                                 ctypes.c_long(K), _p(acc))
    return acc


def matmul_i32_rows(xq, wq, rows):
    """Rows `rows` of the int32 product only -> [len(rows), N]."""
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2 and rows.min() >= 0 and rows.max() < M
    acc = np.empty((rows.size, N), np.int32)
    _load().zq_oracle_matmul_i32_rows(_p(xq), _p(wq), _p(rows), ctypes.c_long(rows.size),
                                      ctypes.c_long(N), ctypes.c_long(K), _p(acc))
    return acc


def matmul_f16_i8(x16, wq, rows=None):
    """FP16 activations x INT8 weight codes in fp64 -> (acc [M,N], absacc [M,N] = sum of |products|).
    `rows` restricts the result to those rows of x."""
    x16 = _c(x16, np.float16)
    wq = _c(wq, np.int8)
    M, K = x16.shape
    N, K2 = wq.shape
    assert K == K2
    r = None
    n_rows = M
    if rows is not None:
        r = np.ascontiguousarray(rows, dtype=np.int64)
        assert r.min() >= 0 and r.max() < M
        n_rows = r.size
    acc = np.empty((n_rows, N), np.float64)
    absacc = np.empty((n_rows, N), np.float64)
    _load().zq_oracle_matmul_f16_i8(_p(x16), _p(wq), None if r is None else _p(r), ctypes.c_long(n_rows),
                                    ctypes.c_long(N), ctypes.c_long(K), _p(acc), _p(absacc))
    return acc, absacc


def dequant_w(acc64, s_w, bias16):
    """Weight-scale-only epilogue in fp64 (no activation scale) -> (ref, mag = |acc*s_w| + |bias|)."""
    acc64 = _c(acc64, np.float64)
    s_w = _c(s_w, np.float32)
    M, N = acc64.shape
    assert N % s_w.size == 0
    ref = np.empty((M, N), np.float64)
    mag = np.empty((M, N), np.float64)
    b = _p(_c(bias16, np.float16)) if bias16 is not None else None
    _load().zq_oracle_dequant_w(_p(acc64), _p(s_w), ctypes.c_long(s_w.size), b, ctypes.c_long(M),
                                ctypes.c_long(N), _p(ref), _p(mag))
    return ref, mag


def dequant(acc, s_tok, s_w, bias16):
    """App. D epilogue in fp64 -> (ref, mag) with mag = |acc*s_tok*s_w| + |bias|."""
    acc = _c(acc, np.int32)
    s_tok = _c(s_tok, np.float32)
    s_w = _c(s_w, np.float32)
    M, N = acc.shape
    assert s_tok.size == M and N % s_w.size == 0
    ref = np.empty((M, N), np.float64)
    mag = np.empty((M, N), np.float64)
    b = _p(_c(bias16, np.float16)) if bias16 is not None else None
    _load().zq_oracle_dequant(_p(acc), _p(s_tok), _p(s_w), ctypes.c_long(s_w.size), b,
                              ctypes.c_long(M), ctypes.c_long(N), _p(ref), _p(mag))
    return ref, mag
