"""ctypes binding of libzq.so: argument marshalling only.

Functions carry the names of the C entry points (include/zq.h) and take torch
CUDA tensors; outputs are allocated here with torch and returned.  The work is
enqueued on torch's current stream.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libzq.so")
_lib = None

SYMBOLS = [
    "zq_status_string", "zq_version", "zq_quantize_weight_groupwise", "zq_layernorm_quant_tokenwise",
    "zq_gelu_quant_tokenwise", "zq_gemm_workspace_bytes", "zq_gemm_i8_dequant", "zq_gemm_w4a8_dequant",
    "zq_debug_force_gemm_variant", "zq_gemm_variant_name", "zq_gemm_choose_variant", "zq_gemm_stream_plan", "zq_gemm_stream_k_ranges", "zq_gemm_gelu_quant_tokenwise", "zq_quantize_tokenwise", "zq_dequantize_acc",
    "zq_tune_set", "zq_tune_clear", "zq_tune_count", "zq_gemm_w8a16_dequant", "zq_gemm_w8a16_workspace_bytes",
    "zq_gemm_w8a16_stream_plan",
    "zq_gemm_quantizes_in_kernel", "zq_debug_set_in_kernel_quant", "zq_quant_wait_expired",
    "zq_workspace_init", "zq_gemm_quant_workspace_bytes", "zq_gemm_i8_dequant_static",
]
PROBE_SYMBOLS = ["zq_probe_read_stream", "zq_probe_mfma_i8", "zq_probe_mfma_i8_tile_traffic"]      # include/zq_probe.h


class ZQError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libzq error %d: %s" % (code, msg))
        self.code = code


def lib_path():
    return _LIB_PATH


def lib():
    """Load libzq.so (built in-tree by paper_2206_01861_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libzq.so is not built; run `python -m paper_2206_01861_amd.build` "
                          "(there is no fallback implementation)")
    L = ctypes.CDLL(_LIB_PATH)
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    L.zq_status_string.restype = ctypes.c_char_p
    L.zq_status_string.argtypes = [ci]
    L.zq_version.restype = ci
    L.zq_version.argtypes = []
    L.zq_quantize_weight_groupwise.restype = ci
    L.zq_quantize_weight_groupwise.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp]
    L.zq_layernorm_quant_tokenwise.restype = ci
    L.zq_layernorm_quant_tokenwise.argtypes = [vp, vp, vp, cf, ci, ci, vp, vp, vp, ci, vp]
    L.zq_gelu_quant_tokenwise.restype = ci
    L.zq_gelu_quant_tokenwise.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, ci, vp]
    L.zq_gemm_workspace_bytes.restype = sz
    L.zq_gemm_workspace_bytes.argtypes = [ci, ci, ci, ci]
    gemm_args = [vp, vp, vp, vp, ci, vp, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    L.zq_gemm_i8_dequant.restype = ci
    L.zq_gemm_i8_dequant.argtypes = gemm_args
    L.zq_gemm_w4a8_dequant.restype = ci
    L.zq_gemm_w4a8_dequant.argtypes = gemm_args
    L.zq_gemm_i8_dequant_static.restype = ci
    L.zq_gemm_i8_dequant_static.argtypes = gemm_args[:13] + [vp]
    L.zq_gemm_gelu_quant_tokenwise.restype = ci
    L.zq_gemm_gelu_quant_tokenwise.argtypes = [vp, vp, vp, ci, vp, ci, vp, ci, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    L.zq_quantize_tokenwise.restype = ci
    L.zq_quantize_tokenwise.argtypes = [vp, ci, ci, vp, vp, vp]
    L.zq_dequantize_acc.restype = ci
    L.zq_dequantize_acc.argtypes = [vp, vp, vp, ci, vp, ci, ci, vp, vp]
    L.zq_gemm_w8a16_dequant.restype = ci
    L.zq_gemm_w8a16_dequant.argtypes = [vp, vp, vp, ci, vp, ci, ci, ci, vp, vp, sz, vp]
    L.zq_tune_set.restype = ci
    L.zq_tune_set.argtypes = [ci] * 8
    L.zq_tune_clear.restype = None
    L.zq_tune_clear.argtypes = []
    L.zq_tune_count.restype = ci
    L.zq_tune_count.argtypes = []
    L.zq_gemm_quantizes_in_kernel.restype = ci
    L.zq_gemm_quantizes_in_kernel.argtypes = [ci, ci, ci, ci, sz]
    L.zq_debug_set_in_kernel_quant.restype = ci
    L.zq_debug_set_in_kernel_quant.argtypes = [ci]
    L.zq_quant_wait_expired.restype = ci
    L.zq_quant_wait_expired.argtypes = [vp, ctypes.POINTER(ci)]
    L.zq_workspace_init.restype = ci
    L.zq_workspace_init.argtypes = [vp, sz, vp]
    L.zq_gemm_quant_workspace_bytes.restype = sz
    L.zq_gemm_quant_workspace_bytes.argtypes = [ci, ci, ci, ci]
    L.zq_debug_force_gemm_variant.restype = ci
    L.zq_debug_force_gemm_variant.argtypes = [ci]
    L.zq_gemm_variant_name.restype = ctypes.c_char_p
    L.zq_gemm_variant_name.argtypes = [ci]
    L.zq_gemm_choose_variant.restype = ci
    L.zq_gemm_choose_variant.argtypes = [ci, ci, ci, ci, sz]
    L.zq_gemm_stream_plan.restype = ci
    L.zq_gemm_stream_plan.argtypes = [ci, ci, ci, ci, sz] + [ctypes.POINTER(ci)] * 3
    L.zq_gemm_stream_k_ranges.restype = ci
    L.zq_gemm_w8a16_workspace_bytes.restype = sz
    L.zq_gemm_w8a16_workspace_bytes.argtypes = [ci, ci, ci]
    L.zq_gemm_w8a16_stream_plan.restype = ci
    L.zq_gemm_w8a16_stream_plan.argtypes = [ci, ci, ci, sz] + [ctypes.POINTER(ci)] * 3
    L.zq_gemm_stream_k_ranges.argtypes = [ci, ci, ci, ci, sz]
    L.zq_probe_read_stream.restype = ci
    L.zq_probe_read_stream.argtypes = [vp, sz, vp, vp]
    L.zq_probe_mfma_i8.restype = ci
    L.zq_probe_mfma_i8.argtypes = [vp, ci, ci, vp, vp]
    L.zq_probe_mfma_i8_tile_traffic.restype = ci
    L.zq_probe_mfma_i8_tile_traffic.argtypes = [vp, sz, ci, ci, vp, vp]
    _lib = L
    return L


def _check(code):
    if code != 0:
        raise ZQError(code, lib().zq_status_string(code).decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (name, dtype))
    return t


def version():
    return lib().zq_version()


def gemm_workspace_bytes(M, N, K, w_bits=8):
    return int(lib().zq_gemm_workspace_bytes(M, N, K, w_bits))


def gemm_quant_workspace_bytes(M, N, K, w_bits=8):
    """Workspace a GeMM call that also quantizes its output can use (zq_gemm_quant_workspace_bytes)."""
    return int(lib().zq_gemm_quant_workspace_bytes(M, N, K, w_bits))


WORKSPACE_FIXED_BYTES = 4227328      # ZQ_WORKSPACE_FIXED_BYTES of include/zq.h


def zq_workspace_init(workspace):
    """Zero the fixed part of a workspace (uint8 CUDA tensor) on torch's current stream."""
    _dev(workspace, torch.uint8, "workspace")
    _check(lib().zq_workspace_init(_ptr(workspace), workspace.numel(), _stream()))
    return workspace


def new_workspace(nbytes, device="cuda"):
    """Allocate (torch) and initialise a workspace of at least nbytes; the smallest legal one if nbytes is less."""
    ws = torch.empty(max(int(nbytes), WORKSPACE_FIXED_BYTES), dtype=torch.uint8, device=device)
    return zq_workspace_init(ws)


def force_gemm_variant(variant):
    """Force a GeMM schedule (-1 = automatic).  Returns the previous setting."""
    return lib().zq_debug_force_gemm_variant(int(variant))


def gemm_variant_name(variant):
    s = lib().zq_gemm_variant_name(int(variant))
    return None if s is None else s.decode()


def gemm_choose_variant(M, N, K, w_bits=8, workspace_bytes=0):
    return lib().zq_gemm_choose_variant(M, N, K, w_bits, workspace_bytes)


def gemm_quantizes_in_kernel(M, N, K, w_bits=8, workspace_bytes=0):
    """True if a GeMM call with quantized output on this shape quantizes inside the GeMM kernel."""
    return bool(lib().zq_gemm_quantizes_in_kernel(M, N, K, w_bits, workspace_bytes))


def set_in_kernel_quant(on):
    """Test/ablation hook (zq_debug_set_in_kernel_quant); returns the previous setting."""
    return bool(lib().zq_debug_set_in_kernel_quant(1 if on else 0))


def quant_wait_expired(workspace):
    """Threads whose bounded wait ran out in calls on this workspace since the last query (0 in a
    correct run).  The caller synchronises first."""
    c = ctypes.c_int(0)
    _check(lib().zq_quant_wait_expired(_ptr(workspace), ctypes.byref(c)))
    return c.value


def tune_set(m_lo, m_hi, N, K, w_bits, variant, row_blocks=0, k_splits=0):
    """Register a measured schedule (and streaming cut) for a shape; see zq_tune_set in include/zq.h."""
    _check(lib().zq_tune_set(m_lo, m_hi, N, K, w_bits, variant, row_blocks, k_splits))


def tune_clear():
    lib().zq_tune_clear()


def tune_count():
    return lib().zq_tune_count()


def gemm_stream_plan(M, N, K, w_bits=8, workspace_bytes=0):
    """(row_blocks, k_splits, consumers) of the weight-streaming schedules for a shape."""
    rb, ks, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().zq_gemm_stream_plan(M, N, K, w_bits, workspace_bytes, ctypes.byref(rb), ctypes.byref(ks),
                                     ctypes.byref(c)))
    return rb.value, ks.value, c.value


def gemm_w8a16_workspace_bytes(M, N, K):
    """Workspace that lets zq_gemm_w8a16_dequant split K for this shape (0: it never splits)."""
    return lib().zq_gemm_w8a16_workspace_bytes(M, N, K)


def gemm_w8a16_stream_plan(M, N, K, workspace_bytes=0):
    """(row_blocks, k_splits, consumers) of the W8A16 streaming schedule (up to 64 tokens)."""
    rb, ks, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().zq_gemm_w8a16_stream_plan(M, N, K, workspace_bytes, ctypes.byref(rb), ctypes.byref(ks),
                                           ctypes.byref(c)))
    return rb.value, ks.value, c.value


def gemm_stream_k_ranges(M, N, K, w_bits=8, workspace_bytes=0):
    """K ranges per strip inside a workgroup of the streaming schedules (1 or 2; 0: shape not taken)."""
    return lib().zq_gemm_stream_k_ranges(M, N, K, w_bits, workspace_bytes)


def zq_probe_read_stream(buf, sink):
    """Read every byte of `buf` (uint8 CUDA tensor, numel % 16 == 0) once; sink: 16-byte CUDA tensor."""
    _dev(buf, torch.uint8, "buf")
    _dev(sink, torch.uint8, "sink")
    _check(lib().zq_probe_read_stream(_ptr(buf), buf.numel(), _ptr(sink), _stream()))


def zq_probe_mfma_i8(operands, blocks, iters, sink):
    """Matrix cores alone (include/zq_probe.h): operands uint8 [blocks*256*128], sink uint8 [blocks*256*16].
    -> number of integer operations the launch performs."""
    _dev(operands, torch.uint8, "operands")
    _dev(sink, torch.uint8, "sink")
    if operands.numel() < blocks * 256 * 128 or sink.numel() < blocks * 256 * 16:
        raise ValueError("operands / sink too small for %d blocks" % blocks)
    _check(lib().zq_probe_mfma_i8(_ptr(operands), blocks, iters, _ptr(sink), _stream()))
    return blocks * 4 * iters * 16 * 65536


def zq_probe_mfma_i8_tile_traffic(source, blocks, iters, sink):
    """Matrix cores with the operand traffic of the 256x256 tile (include/zq_probe.h): source uint8, at least
    2 MiB; sink uint8 [blocks*512*16].  -> number of integer operations the launch performs."""
    _dev(source, torch.uint8, "source")
    _dev(sink, torch.uint8, "sink")
    if source.numel() < (2 << 20) or sink.numel() < blocks * 512 * 16:
        raise ValueError("source / sink too small for %d blocks" % blocks)
    _check(lib().zq_probe_mfma_i8_tile_traffic(_ptr(source), source.numel(), blocks, iters, _ptr(sink), _stream()))
    return blocks * 8 * iters * 32 * 65536


def zq_quantize_weight_groupwise(w_fp16, groups, bits):
    """w fp16 [N,K] -> (wq int8 [N,K] | uint8 [N,K/2], s_w fp32 [groups])."""
    _dev(w_fp16, torch.float16, "w_fp16")
    N, K = w_fp16.shape
    if bits == 4:
        wq = torch.empty((N, K // 2), dtype=torch.uint8, device=w_fp16.device)
    else:
        wq = torch.empty((N, K), dtype=torch.int8, device=w_fp16.device)
    s_w = torch.empty(max(groups, 1), dtype=torch.float32, device=w_fp16.device)
    _check(lib().zq_quantize_weight_groupwise(_ptr(w_fp16), N, K, groups, bits, _ptr(wq), _ptr(s_w), _stream()))
    return wq, s_w


def _y_buf(M, K, y_dtype, device):
    if y_dtype is None:
        return None, 0
    if y_dtype == torch.float32:
        return torch.empty((M, K), dtype=torch.float32, device=device), 1
    if y_dtype == torch.float16:
        return torch.empty((M, K), dtype=torch.float16, device=device), 0
    raise TypeError("y_dtype must be None, torch.float16 or torch.float32")


def zq_layernorm_quant_tokenwise(x_fp16, gamma_fp16, beta_fp16, eps, y_dtype=None, out=None):
    """x fp16 [M,K] -> (xq int8 [M,K], s_tok fp32 [M], y or None)."""
    _dev(x_fp16, torch.float16, "x_fp16")
    _dev(gamma_fp16, torch.float16, "gamma_fp16")
    if beta_fp16 is not None:
        _dev(beta_fp16, torch.float16, "beta_fp16")
    M, K = x_fp16.shape
    xq, s_tok = out if out is not None else (
        torch.empty((M, K), dtype=torch.int8, device=x_fp16.device),
        torch.empty(M, dtype=torch.float32, device=x_fp16.device))
    y, yd = _y_buf(M, K, y_dtype, x_fp16.device)
    _check(lib().zq_layernorm_quant_tokenwise(_ptr(x_fp16), _ptr(gamma_fp16), _ptr(beta_fp16), float(eps), M, K,
                                              _ptr(xq), _ptr(s_tok), _ptr(y), yd, _stream()))
    return xq, s_tok, y


def zq_gelu_quant_tokenwise(h_fp16, bias_fp16=None, approx_tanh=False, y_dtype=None, out=None):
    """h fp16 [M,N] -> (xq int8 [M,N], s_tok fp32 [M], y or None)."""
    _dev(h_fp16, torch.float16, "h_fp16")
    if bias_fp16 is not None:
        _dev(bias_fp16, torch.float16, "bias_fp16")
    M, N = h_fp16.shape
    xq, s_tok = out if out is not None else (
        torch.empty((M, N), dtype=torch.int8, device=h_fp16.device),
        torch.empty(M, dtype=torch.float32, device=h_fp16.device))
    y, yd = _y_buf(M, N, y_dtype, h_fp16.device)
    _check(lib().zq_gelu_quant_tokenwise(_ptr(h_fp16), _ptr(bias_fp16), 1 if approx_tanh else 0, M, N,
                                         _ptr(xq), _ptr(s_tok), _ptr(y), yd, _stream()))
    return xq, s_tok, y


def _out_shape(t, M, N, name):
    if tuple(t.shape) != (M, N):
        raise ValueError("%s must be [%d, %d], got %s" % (name, M, N, tuple(t.shape)))


def _gemm_shapes(M, N, K, wq, w_bits, s_tok, bias_fp16):
    """The C ABI trusts the sizes it is given: check every tensor against (M, N, K) before the call."""
    if wq.dim() != 2 or wq.shape[1] * (8 // w_bits) != K:
        raise ValueError("wq must be [N, %s] for K = %d, got %s" % ("K" if w_bits == 8 else "K/2", K, tuple(wq.shape)))
    if s_tok is not None and s_tok.numel() != M:
        raise ValueError("s_tok must hold %d scales, got %d" % (M, s_tok.numel()))
    if bias_fp16 is not None and bias_fp16.numel() != N:
        raise ValueError("bias must hold %d values, got %d" % (N, bias_fp16.numel()))


def _ws_bytes(workspace):
    if workspace is None:
        return 0
    _dev(workspace, torch.uint8, "workspace")
    return workspace.numel()


def _gemm(fn, wdtype, xq, s_tok, wq, s_w, bias_fp16, want_acc, requant, workspace, out, acc_out=None):
    _dev(xq, torch.int8, "xq")
    _dev(s_tok, torch.float32, "s_tok")
    _dev(wq, wdtype, "wq")
    _dev(s_w, torch.float32, "s_w")
    if bias_fp16 is not None:
        _dev(bias_fp16, torch.float16, "bias_fp16")
    M, K = xq.shape
    N = wq.shape[0]
    _gemm_shapes(M, N, K, wq, 8 if wdtype == torch.int8 else 4, s_tok, bias_fp16)
    dev = xq.device
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=dev)
    _out_shape(_dev(out, torch.float16, "out"), M, N, "out")
    acc = acc_out if acc_out is not None else (torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None)
    if acc is not None:
        _out_shape(_dev(acc, torch.int32, "acc_out"), M, N, "acc_out")
    out_q = torch.empty((M, N), dtype=torch.int8, device=dev) if requant else None
    out_s = torch.empty(M, dtype=torch.float32, device=dev) if requant else None
    ws_bytes = _ws_bytes(workspace)
    _check(fn(_ptr(xq), _ptr(s_tok), _ptr(wq), _ptr(s_w), int(s_w.numel()), _ptr(bias_fp16), M, N, K, _ptr(out),
              _ptr(acc), _ptr(out_q), _ptr(out_s), _ptr(workspace), ws_bytes, _stream()))
    return out, acc, out_q, out_s


def zq_gemm_i8_dequant(xq, s_tok, wq, s_w, bias_fp16=None, want_acc=False, requant=False, workspace=None,
                       out=None, acc_out=None):
    """-> (out fp16 [M,N], acc int32 | None, out_q int8 | None, out_s_tok fp32 | None)."""
    return _gemm(lib().zq_gemm_i8_dequant, torch.int8, xq, s_tok, wq, s_w, bias_fp16, want_acc, requant,
                 workspace, out, acc_out)


STATIC_SCRATCH_BYTES = 16777216      # ZQ_STATIC_SCRATCH_BYTES of include/zq.h


def zq_gemm_i8_dequant_static(xq, s_tok, wq, s_w, bias_fp16=None, requant=False, out=None, acc_out=None,
                              out_q=None, out_s_tok=None):
    """zq_gemm_i8_dequant on the library's static scratch buffer: the C call allocates nothing, and
    neither does this wrapper when out (and acc_out, out_q, out_s_tok as wanted) are passed in.
    -> (out, acc_out, out_q, out_s_tok)."""
    _dev(xq, torch.int8, "xq")
    _dev(s_tok, torch.float32, "s_tok")
    _dev(wq, torch.int8, "wq")
    _dev(s_w, torch.float32, "s_w")
    if bias_fp16 is not None:
        _dev(bias_fp16, torch.float16, "bias_fp16")
    M, K = xq.shape
    N = wq.shape[0]
    _gemm_shapes(M, N, K, wq, 8, s_tok, bias_fp16)
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _out_shape(_dev(out, torch.float16, "out"), M, N, "out")
    if acc_out is not None:
        _out_shape(_dev(acc_out, torch.int32, "acc_out"), M, N, "acc_out")
    if requant and out_q is None:
        out_q = torch.empty((M, N), dtype=torch.int8, device=xq.device)
        out_s_tok = torch.empty(M, dtype=torch.float32, device=xq.device)
    if out_q is not None:
        _out_shape(_dev(out_q, torch.int8, "out_q"), M, N, "out_q")
        if _dev(out_s_tok, torch.float32, "out_s_tok").numel() != M:
            raise ValueError("out_s_tok must hold %d scales" % M)
    _check(lib().zq_gemm_i8_dequant_static(_ptr(xq), _ptr(s_tok), _ptr(wq), _ptr(s_w), int(s_w.numel()),
                                           _ptr(bias_fp16), M, N, K, _ptr(out), _ptr(acc_out), _ptr(out_q),
                                           _ptr(out_s_tok), _stream()))
    return out, acc_out, out_q, out_s_tok


def zq_gemm_w4a8_dequant(xq, s_tok, wq4, s_w, bias_fp16=None, want_acc=False, requant=False, workspace=None,
                         out=None, acc_out=None):
    """INT4-packed weights uint8 [N,K/2]; otherwise as zq_gemm_i8_dequant."""
    return _gemm(lib().zq_gemm_w4a8_dequant, torch.uint8, xq, s_tok, wq4, s_w, bias_fp16, want_acc, requant,
                 workspace, out, acc_out)


def zq_gemm_gelu_quant_tokenwise(xq, s_tok, wq, s_w, bias_fp16=None, approx_tanh=False, workspace=None, out=None,
                                 keep_g=True):
    """GeMM with bias + GeLU in its epilogue, then token-wise INT8 quantization of the FP16 result.

    wq int8 [N,K] or INT4-packed uint8 [N,K/2].  -> (g fp16 [M,N], gq int8 [M,N], s_tok fp32 [M]);
    `out` = (g, gq, s) reuses caller tensors.  keep_g=False passes no g buffer (g comes back None):
    allowed where gemm_quantizes_in_kernel() holds, an error elsewhere.
    """
    _dev(xq, torch.int8, "xq")
    _dev(s_tok, torch.float32, "s_tok")
    _dev(s_w, torch.float32, "s_w")
    if wq.dtype == torch.int8:
        w_bits = 8
    elif wq.dtype == torch.uint8:
        w_bits = 4
        if wq.shape[1] * 2 != xq.shape[1]:
            raise ValueError("wq4 must be [N, K/2]")
    else:
        raise TypeError("wq must be int8 (INT8) or uint8 (packed INT4)")
    _dev(wq, wq.dtype, "wq")
    if bias_fp16 is not None:
        _dev(bias_fp16, torch.float16, "bias_fp16")
    M, K = xq.shape
    N = wq.shape[0]
    _gemm_shapes(M, N, K, wq, w_bits, s_tok, bias_fp16)
    dev = xq.device
    g, gq, s = out if out is not None else (
        torch.empty((M, N), dtype=torch.float16, device=dev) if keep_g else None,
        torch.empty((M, N), dtype=torch.int8, device=dev),
        torch.empty(M, dtype=torch.float32, device=dev))
    if not keep_g:
        g = None
    if g is not None:
        _out_shape(_dev(g, torch.float16, "g"), M, N, "g")
    _out_shape(_dev(gq, torch.int8, "gq"), M, N, "gq")
    if _dev(s, torch.float32, "s_tok_out").numel() != M:
        raise ValueError("s_tok_out must hold %d scales" % M)
    ws_bytes = _ws_bytes(workspace)
    _check(lib().zq_gemm_gelu_quant_tokenwise(_ptr(xq), _ptr(s_tok), _ptr(wq), w_bits, _ptr(s_w), int(s_w.numel()),
                                              _ptr(bias_fp16), 1 if approx_tanh else 0, M, N, K, _ptr(g), _ptr(gq),
                                              _ptr(s), _ptr(workspace), ws_bytes, _stream()))
    return g, gq, s


def zq_quantize_tokenwise(x_fp16, out=None):
    """x fp16 [M,K] -> (xq int8 [M,K], s_tok fp32 [M])."""
    _dev(x_fp16, torch.float16, "x_fp16")
    M, K = x_fp16.shape
    xq, s_tok = out if out is not None else (
        torch.empty((M, K), dtype=torch.int8, device=x_fp16.device),
        torch.empty(M, dtype=torch.float32, device=x_fp16.device))
    _check(lib().zq_quantize_tokenwise(_ptr(x_fp16), M, K, _ptr(xq), _ptr(s_tok), _stream()))
    return xq, s_tok


def zq_dequantize_acc(acc, s_tok, s_w, bias_fp16=None, out=None):
    """acc int32 [M,N] -> fp16 [M,N] = acc * s_tok[row] * s_w[group] + bias."""
    _dev(acc, torch.int32, "acc")
    _dev(s_tok, torch.float32, "s_tok")
    _dev(s_w, torch.float32, "s_w")
    if bias_fp16 is not None:
        _dev(bias_fp16, torch.float16, "bias_fp16")
    M, N = acc.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=acc.device)
    _check(lib().zq_dequantize_acc(_ptr(acc), _ptr(s_tok), _ptr(s_w), int(s_w.numel()), _ptr(bias_fp16), M, N,
                                   _ptr(out), _stream()))
    return out


def zq_gemm_w8a16_dequant(x_fp16, wq, s_w, bias_fp16=None, workspace=None, out=None):
    """x fp16 [M,K] x wq int8 [N,K] -> out fp16 [M,N] = (x @ wq^T) * s_w[group] + bias."""
    _dev(x_fp16, torch.float16, "x_fp16")
    _dev(wq, torch.int8, "wq")
    _dev(s_w, torch.float32, "s_w")
    if bias_fp16 is not None:
        _dev(bias_fp16, torch.float16, "bias_fp16")
    M, K = x_fp16.shape
    N = wq.shape[0]
    _gemm_shapes(M, N, K, wq, 8, None, bias_fp16)
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x_fp16.device)
    _out_shape(_dev(out, torch.float16, "out"), M, N, "out")
    ws_bytes = _ws_bytes(workspace)
    _check(lib().zq_gemm_w8a16_dequant(_ptr(x_fp16), _ptr(wq), _ptr(s_w), int(s_w.numel()), _ptr(bias_fp16), M, N, K,
                                       _ptr(out), _ptr(workspace), ws_bytes, _stream()))
    return out
