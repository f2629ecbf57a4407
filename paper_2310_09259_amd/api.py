"""Thin Python binding of the C ABI in include/quik.h (argument marshalling only).

torch is used for device memory and for the current HIP stream; every step of
the layer runs in the library's own kernels.  There is no CPU fallback: if the
shared library is missing, loading it raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libquik.so")

_lib = None


class QuikError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def load() -> C.CDLL:
    """Load libquik.so (built in-tree by paper_2310_09259_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2310_09259_amd.build` "
                "(there is no fallback path)")
        lib = C.CDLL(LIB_PATH)
        vp, i, f = C.c_void_p, C.c_int, C.c_void_p
        lib.quik_version.restype = i
        lib.quik_status_string.restype = C.c_char_p
        lib.quik_status_string.argtypes = [i]
        lib.quik_packed_row_bytes.restype = i
        lib.quik_packed_row_bytes.argtypes = [i, i]
        lib.quik_workspace_bytes.restype = C.c_size_t
        lib.quik_workspace_bytes.argtypes = [i, i, i, i, i]
        lib.quik_workspace_regions.restype = i
        lib.quik_workspace_regions.argtypes = [i, i, i, i, i, vp, vp]
        lib.quik_debug_gemm_plan.restype = i
        lib.quik_debug_gemm_plan.argtypes = [i, i, i, i, vp]
        lib.quik_debug_gemm_tile.restype = i
        lib.quik_debug_gemm_tile.argtypes = [i, i, i, i, i, i, vp]
        lib.quik_debug_set_gemm_path.restype = i
        lib.quik_debug_set_gemm_path.argtypes = [i]
        lib.quik_quantize_workspace_bytes.restype = C.c_size_t
        lib.quik_quantize_workspace_bytes.argtypes = [i, i]
        lib.quik_w_reduced_bytes.restype = C.c_size_t
        lib.quik_w_reduced_bytes.argtypes = [i, i]
        lib.quik_quantize.restype = i
        lib.quik_quantize.argtypes = [vp, i, i, i, vp, i, i, vp, i, f, f, vp, i, vp, C.c_size_t, vp]
        lib.quik_weight_reduce.restype = i
        lib.quik_weight_reduce.argtypes = [vp, i, vp, i, i, i, f, vp]
        lib.quik_gemm_dequant.restype = i
        lib.quik_gemm_dequant.argtypes = [vp, i, f, f, vp, i, i, i, i, i, vp, i, vp, f, vp, i,
                                          vp, i, vp, i, vp, C.c_size_t, vp]
        for fn in (lib.quik_debug_int_gemm, lib.quik_int_gemm):
            fn.restype = i
            fn.argtypes = [vp, i, vp, i, i, i, i, i, vp, i, vp, C.c_size_t, vp, vp]
        lib.quik_linear.restype = i
        lib.quik_linear.argtypes = [vp, i, i, i, vp, i, i, vp, i, vp, f, vp, i, vp, i, vp, i, vp,
                                    C.c_size_t, vp]
        lib.quik_linear_noalloc.restype = i
        lib.quik_linear_noalloc.argtypes = [vp, i, i, i, vp, i, i, vp, i, vp, f, vp, i, vp, i, vp, i, vp]
        lib.quik_ablation_workspace_bytes.restype = C.c_size_t
        lib.quik_ablation_workspace_bytes.argtypes = [i, i, i, i, i]
        lib.quik_linear_ablation.restype = i
        lib.quik_linear_ablation.argtypes = [i, vp, i, i, i, vp, i, i, vp, i, vp, f, vp, i, vp, i, vp, i,
                                             vp, C.c_size_t, vp]
        lib.quik_gemm_dequant_w4a8.restype = i
        lib.quik_gemm_dequant_w4a8.argtypes = [vp, i, f, f, vp, i, i, i, i, vp, i, vp, f, vp, i, vp, i, vp, i, vp]
        lib.quik_int_gemm_w4a8.restype = i
        lib.quik_int_gemm_w4a8.argtypes = [vp, i, vp, i, i, i, i, vp, i, vp]
        lib.quik_linear_w4a8.restype = i
        lib.quik_linear_w4a8.argtypes = [vp, i, i, i, vp, i, vp, i, vp, f, vp, i, vp, i, vp, i, vp,
                                         C.c_size_t, vp]
        lib.quik_fp6_row_bytes.restype = i
        lib.quik_fp6_row_bytes.argtypes = [i]
        lib.quik_workspace_bytes_fp6.restype = C.c_size_t
        lib.quik_workspace_bytes_fp6.argtypes = [i, i, i, i]
        lib.quik_weight_pack_fp6.restype = i
        lib.quik_weight_pack_fp6.argtypes = [vp, i, i, i, vp, vp]
        lib.quik_quantize_fp6.restype = i
        lib.quik_quantize_fp6.argtypes = [vp, i, i, i, vp, i, vp, f, f, vp, i, vp]
        lib.quik_gemm_dequant_fp6.restype = i
        lib.quik_gemm_dequant_fp6.argtypes = [vp, f, f, vp, i, i, i, i, vp, vp, f, vp, i, vp, i, vp, i, vp]
        lib.quik_int_gemm_fp6.restype = i
        lib.quik_int_gemm_fp6.argtypes = [vp, vp, i, i, i, vp, i, vp]
        lib.quik_sp24_act_row_bytes.restype = i
        lib.quik_sp24_act_row_bytes.argtypes = [i]
        lib.quik_sp24_weight_bytes.restype = C.c_size_t
        lib.quik_sp24_weight_bytes.argtypes = [i, i]
        lib.quik_workspace_bytes_sp24.restype = C.c_size_t
        lib.quik_workspace_bytes_sp24.argtypes = [i, i, i, i]
        lib.quik_weight_pack_sp24.restype = i
        lib.quik_weight_pack_sp24.argtypes = [vp, i, i, i, vp, vp, vp]
        lib.quik_quantize_sp24.restype = i
        lib.quik_quantize_sp24.argtypes = [vp, i, i, i, vp, i, vp, f, f, vp, i, vp]
        lib.quik_gemm_dequant_sp24.restype = i
        lib.quik_gemm_dequant_sp24.argtypes = [vp, f, f, vp, i, i, i, i, vp, vp, f, vp, i, vp, i, vp, i, vp]
        lib.quik_int_gemm_sp24.restype = i
        lib.quik_int_gemm_sp24.argtypes = [vp, vp, i, i, i, vp, i, vp]
        lib.quik_linear_sp24.restype = i
        lib.quik_linear_sp24.argtypes = [vp, i, i, i, vp, i, vp, vp, f, vp, i, vp, i, vp, i, vp, C.c_size_t, vp]
        lib.quik_linear_fp6.restype = i
        lib.quik_linear_fp6.argtypes = [vp, i, i, i, vp, i, vp, vp, f, vp, i, vp, i, vp, i, vp, C.c_size_t, vp]
        lib.quik_debug_mfma_probe.restype = i
        lib.quik_debug_mfma_probe.argtypes = [i, i, vp, vp]
        lib.quik_debug_mix_probe.restype = i
        lib.quik_debug_mix_probe.argtypes = [i, i, i, vp, vp, C.c_size_t, vp, vp]
        lib.quik_debug_copy_probe.restype = i
        lib.quik_debug_copy_probe.argtypes = [vp, vp, C.c_size_t, vp]
        lib.quik_check_outlier_idx_host.restype = i
        lib.quik_check_outlier_idx_host.argtypes = [vp, i, i]
        _lib = lib
    return _lib


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise QuikError(rc, where)


def _dev(t, dtype, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if t.dim() > 1 and t.stride(-1) != 1:
        raise ValueError(f"{name} must be contiguous along its last dimension")
    return t


def quik_version() -> int:
    return load().quik_version()


def status_string(status: int) -> str:
    return load().quik_status_string(status).decode()


def quik_packed_row_bytes(K_b: int, bits: int) -> int:
    return load().quik_packed_row_bytes(K_b, bits)


def quik_workspace_bytes(T: int, K: int, N: int, n_out: int, bits: int) -> int:
    return load().quik_workspace_bytes(T, K, N, n_out, bits)


def quik_debug_mfma_probe(workgroups: int, iters: int, sink):
    """Enqueue the int8 matrix-instruction probe; returns the integer operations it performs."""
    _check(load().quik_debug_mfma_probe(workgroups, iters, _ptr(sink), _stream()), "quik_debug_mfma_probe")
    return 2.0 * 32 * 32 * 32 * 16 * workgroups * iters


def quik_debug_mix_probe(mix: int, workgroups: int, iters: int, sink, src=None, clocks=None):
    """Enqueue the K-loop instruction-mix probe (see include/quik.h for the bits of `mix`); returns the
    integer operations it performs.  clocks: int64 device tensor [2] or None."""
    _check(load().quik_debug_mix_probe(mix, workgroups, iters, _ptr(sink), _ptr(src), _nbytes(src), _ptr(clocks),
                                       _stream()), "quik_debug_mix_probe")
    return 2.0 * 32 * 32 * 32 * 12 * 8 * workgroups * iters


def quik_debug_copy_probe(src, dst):
    """Enqueue a plain streaming copy src -> dst (uint8 device tensors of equal size)."""
    _check(load().quik_debug_copy_probe(_ptr(src), _ptr(dst), src.numel(), _stream()), "quik_debug_copy_probe")


def quik_check_outlier_idx_host(idx_host, K: int) -> int:
    import numpy as np
    a = np.ascontiguousarray(idx_host, dtype=np.int32)
    return load().quik_check_outlier_idx_host(a.ctypes.data_as(C.c_void_p), int(a.size), K)


def quik_debug_gemm_plan(T: int, N: int, K_b: int, cus: int):
    """Host-only: None if the persistent 4-bit kernel cannot run this shape on `cus` compute units, else
    (choice, (tiles_m, tn, base, rem, grid)): choice 1 = it is used, 2 = the per-tile kernels are."""
    plan = (C.c_int * 5)()
    rc = load().quik_debug_gemm_plan(T, N, K_b, cus, C.cast(plan, C.c_void_p))
    if rc < 0:
        _check(rc, "quik_debug_gemm_plan")
    return (rc, tuple(plan)) if rc > 0 else None


def quik_debug_set_gemm_path(mode: int):
    """0 automatic, 1 persistent 4-bit kernel wherever it can run, 2 per-tile kernels only."""
    _check(load().quik_debug_set_gemm_path(mode), "quik_debug_set_gemm_path")


def quik_quantize_workspace_bytes(T: int, bits: int) -> int:
    return load().quik_quantize_workspace_bytes(T, bits)


def quik_w_reduced_bytes(N: int, bits: int) -> int:
    return load().quik_w_reduced_bytes(N, bits)


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def quik_quantize(x, outlier_idx, bits: int, out=None):
    """x fp16 [T,K] -> (xq uint8 [T,ldq], scale f32 [T], zero f32 [T], x_out f16 [T,n_out],
    workspace uint8 [quik_quantize_workspace_bytes]).  The workspace carries the side data that
    quik_gemm_dequant needs beside xq for bits = 4."""
    x = _dev(x, torch.float16, "x")
    T, K = x.shape
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    if n_out:
        _dev(outlier_idx, torch.int32, "outlier_idx")
    K_b = K - n_out
    ldq = quik_packed_row_bytes(K_b, bits)
    if ldq <= 0:
        raise QuikError(-1, "quik_packed_row_bytes")
    if out is None:
        xq = torch.empty((T, ldq), dtype=torch.uint8, device=x.device)
        scale = torch.empty(T, dtype=torch.float32, device=x.device)
        zero = torch.empty(T, dtype=torch.float32, device=x.device)
        x_out = torch.empty((T, n_out), dtype=torch.float16, device=x.device)
        side = torch.empty(quik_quantize_workspace_bytes(T, bits), dtype=torch.uint8, device=x.device)
    else:
        xq, scale, zero, x_out, side = out
    rc = load().quik_quantize(_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out,
                              bits, _ptr(xq), xq.stride(0), _ptr(scale), _ptr(zero),
                              _ptr(x_out) if n_out else None, x_out.stride(0) if n_out else 0,
                              _ptr(side), _nbytes(side), _stream())
    _check(rc, "quik_quantize")
    return xq, scale, zero, x_out, side


def quik_weight_reduce(w_q, w_scale, K_b: int, bits: int):
    """-> w_reduced f32 [quik_w_reduced_bytes / 4]: wReduced in the first N entries (for bits = 4
    followed by N entries of side data for the 4-bit GEMM)."""
    w_q = _dev(w_q, torch.uint8, "w_q")
    w_scale = _dev(w_scale, torch.float16, "w_scale")
    N = w_q.shape[0]
    out = torch.empty(quik_w_reduced_bytes(N, bits) // 4, dtype=torch.float32, device=w_q.device)
    rc = load().quik_weight_reduce(_ptr(w_q), w_q.stride(0), _ptr(w_scale), N, K_b, bits, _ptr(out), _stream())
    _check(rc, "quik_weight_reduce")
    return out


def _gemm_dequant_args(xq, scale, zero, x_out, K_b, bits, w_q, w_scale, w_reduced, w_out, bias, y, workspace):
    T, N = xq.shape[0], w_q.shape[0]
    n_out = 0 if x_out is None else int(x_out.shape[1])
    return (_ptr(xq), xq.stride(0), _ptr(scale), _ptr(zero), _ptr(x_out) if n_out else None,
            x_out.stride(0) if n_out else 0, T, K_b, n_out, bits, _ptr(w_q), w_q.stride(0), _ptr(w_scale),
            _ptr(w_reduced), _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0, _ptr(bias), N,
            _ptr(y), y.stride(0), _ptr(workspace), _nbytes(workspace), _stream())


def quik_gemm_dequant(xq, scale, zero, x_out, K_b: int, bits: int, w_q, w_scale, w_reduced, w_out, bias=None,
                      out=None, workspace=None):
    """workspace: the one quik_quantize returned together with xq (needed for bits = 4)."""
    xq = _dev(xq, torch.uint8, "xq")
    w_q = _dev(w_q, torch.uint8, "w_q")
    T, N = xq.shape[0], w_q.shape[0]
    n_out = 0 if x_out is None else int(x_out.shape[1])
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=xq.device)
    rc = load().quik_gemm_dequant(*_gemm_dequant_args(xq, scale, zero, x_out, K_b, bits, w_q, w_scale, w_reduced,
                                                      w_out, bias, y, workspace))
    _check(rc, "quik_gemm_dequant")
    return y


def quik_debug_int_gemm(xq, w_q, K_b: int, bits: int, workspace=None, w_reduced=None):
    """Raw INT32 accumulators.  workspace (from quik_quantize) and w_reduced (from quik_weight_reduce)
    together select the fused kernel's operand widening; neither: the widening without side data."""
    xq = _dev(xq, torch.uint8, "xq")
    w_q = _dev(w_q, torch.uint8, "w_q")
    T, N = xq.shape[0], w_q.shape[0]
    acc = torch.empty((T, N), dtype=torch.int32, device=xq.device)
    rc = load().quik_debug_int_gemm(_ptr(xq), xq.stride(0), _ptr(w_q), w_q.stride(0), T, N, K_b, bits,
                                    _ptr(acc), acc.stride(0), _ptr(workspace), _nbytes(workspace),
                                    _ptr(w_reduced), _stream())
    _check(rc, "quik_debug_int_gemm")
    return acc


quik_int_gemm = quik_debug_int_gemm


def _linear_buffers(x, outlier_idx, bits, w_q, out, workspace):
    x = _dev(x, torch.float16, "x")
    w_q = _dev(w_q, torch.uint8, "w_q")
    T, K = x.shape
    N = w_q.shape[0]
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    need = quik_workspace_bytes(T, K, N, n_out, bits)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=x.device)
    return y, workspace


def _linear_args(x, outlier_idx, bits, w_q, w_scale, w_reduced, w_out, bias, y, workspace):
    T, K = x.shape
    N = w_q.shape[0]
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    return (_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, bits, _ptr(w_q),
            w_q.stride(0), _ptr(w_scale), _ptr(w_reduced), _ptr(w_out) if n_out else None,
            w_out.stride(0) if n_out else 0, _ptr(bias), N, _ptr(y), y.stride(0), _ptr(workspace),
            _nbytes(workspace), _stream())


def quik_linear(x, outlier_idx, bits: int, w_q, w_scale, w_reduced, w_out, bias=None, out=None, workspace=None):
    """Whole layer.  Returns y fp16 [T, N]."""
    y, workspace = _linear_buffers(x, outlier_idx, bits, w_q, out, workspace)
    rc = load().quik_linear(*_linear_args(x, outlier_idx, bits, w_q, w_scale, w_reduced, w_out, bias, y, workspace))
    _check(rc, "quik_linear")
    return y


def quik_linear_noalloc(x, outlier_idx, bits: int, w_q, w_scale, w_reduced, w_out, out, bias=None):
    """quik_linear without a workspace argument (the library's static device array holds the
    intermediate results).  `out` (fp16 [T, N]) is required: the call itself allocates nothing."""
    x = _dev(x, torch.float16, "x")
    w_q = _dev(w_q, torch.uint8, "w_q")
    y = _dev(out, torch.float16, "out")
    args = _linear_args(x, outlier_idx, bits, w_q, w_scale, w_reduced, w_out, bias, y, None)
    rc = load().quik_linear_noalloc(*args[:-3], args[-1])
    _check(rc, "quik_linear_noalloc")
    return y


def prepare_linear(x, outlier_idx, bits: int, w_q, w_scale, w_reduced, w_out, bias=None, out=None,
                   workspace=None):
    """quik_linear with the argument marshalling done once: returns (call, y) where call() enqueues
    one layer on the stream that was current here, on the same buffers every time.  For loops that
    launch the same layer many times (serving, benchmarking), where building the ctypes arguments
    would otherwise cost more host time than a small layer takes on the GPU."""
    y, workspace = _linear_buffers(x, outlier_idx, bits, w_q, out, workspace)
    args = _linear_args(x, outlier_idx, bits, w_q, w_scale, w_reduced, w_out, bias, y, workspace)
    keep = (x, outlier_idx, w_q, w_scale, w_reduced, w_out, bias, y, workspace)
    return _prepared(load().quik_linear, "quik_linear", args, keep), y


def quik_gemm_dequant_w4a8(xq, scale, zero, x_out, K_b: int, w_q, w_scale, w_reduced, w_out, bias=None,
                           out=None):
    """8-bit activations (quik_quantize with bits=8) times packed 4-bit weights."""
    xq = _dev(xq, torch.uint8, "xq")
    w_q = _dev(w_q, torch.uint8, "w_q")
    T, N = xq.shape[0], w_q.shape[0]
    n_out = 0 if x_out is None else int(x_out.shape[1])
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=xq.device)
    rc = load().quik_gemm_dequant_w4a8(
        _ptr(xq), xq.stride(0), _ptr(scale), _ptr(zero), _ptr(x_out) if n_out else None,
        x_out.stride(0) if n_out else 0, T, K_b, n_out, _ptr(w_q), w_q.stride(0), _ptr(w_scale),
        _ptr(w_reduced), _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0, _ptr(bias), N,
        _ptr(y), y.stride(0), _stream())
    _check(rc, "quik_gemm_dequant_w4a8")
    return y


def quik_int_gemm_w4a8(xq, w_q, K_b: int):
    xq = _dev(xq, torch.uint8, "xq")
    w_q = _dev(w_q, torch.uint8, "w_q")
    T, N = xq.shape[0], w_q.shape[0]
    acc = torch.empty((T, N), dtype=torch.int32, device=xq.device)
    rc = load().quik_int_gemm_w4a8(_ptr(xq), xq.stride(0), _ptr(w_q), w_q.stride(0), T, N, K_b, _ptr(acc),
                                   acc.stride(0), _stream())
    _check(rc, "quik_int_gemm_w4a8")
    return acc


def quik_linear_w4a8(x, outlier_idx, w_q, w_scale, w_reduced, w_out, bias=None, out=None, workspace=None):
    """Whole layer with 8-bit activations and packed 4-bit weights.  Returns y fp16 [T, N]."""
    x = _dev(x, torch.float16, "x")
    w_q = _dev(w_q, torch.uint8, "w_q")
    T, K = x.shape
    N = w_q.shape[0]
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    need = quik_workspace_bytes(T, K, N, n_out, 8)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=x.device)
    rc = load().quik_linear_w4a8(
        _ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, _ptr(w_q), w_q.stride(0),
        _ptr(w_scale), _ptr(w_reduced), _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0,
        _ptr(bias), N, _ptr(y), y.stride(0), _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "quik_linear_w4a8")
    return y


def _prepared(fn, name, args, keep):
    def call(_keep=keep):
        rc = fn(*args)
        if rc != 0:
            raise QuikError(rc, name)
    return call


def prepare_linear_w4a8(x, outlier_idx, w_q, w_scale, w_reduced, w_out, bias=None, out=None, workspace=None):
    """Marshal-once form of quik_linear_w4a8: returns (call, y)."""
    x = _dev(x, torch.float16, "x")
    w_q = _dev(w_q, torch.uint8, "w_q")
    T, K = x.shape
    N = w_q.shape[0]
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    need = quik_workspace_bytes(T, K, N, n_out, 8)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=x.device)
    args = (_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, _ptr(w_q), w_q.stride(0),
            _ptr(w_scale), _ptr(w_reduced), _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0,
            _ptr(bias), N, _ptr(y), y.stride(0), _ptr(workspace), workspace.numel(), _stream())
    keep = (x, outlier_idx, w_q, w_scale, w_reduced, w_out, bias, y, workspace)
    return _prepared(load().quik_linear_w4a8, "quik_linear_w4a8", args, keep), y


def prepare_quantize(x, outlier_idx, bits: int, out):
    """Marshal-once form of quik_quantize writing into out = (xq, scale, zero, x_out, workspace)."""
    x = _dev(x, torch.float16, "x")
    T, K = x.shape
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    xq, scale, zero, x_out, side = out
    args = (_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, bits, _ptr(xq),
            xq.stride(0), _ptr(scale), _ptr(zero), _ptr(x_out) if n_out else None,
            x_out.stride(0) if n_out else 0, _ptr(side), _nbytes(side), _stream())
    return _prepared(load().quik_quantize, "quik_quantize", args, (x, outlier_idx, out))


def prepare_gemm_dequant(xq, scale, zero, x_out, K_b: int, bits: int, w_q, w_scale, w_reduced, w_out, bias, out,
                         workspace):
    """Marshal-once form of quik_gemm_dequant writing into `out`."""
    args = _gemm_dequant_args(xq, scale, zero, x_out, K_b, bits, w_q, w_scale, w_reduced, w_out, bias, out,
                              workspace)
    keep = (xq, scale, zero, x_out, w_q, w_scale, w_reduced, w_out, bias, out, workspace)
    return _prepared(load().quik_gemm_dequant, "quik_gemm_dequant", args, keep)


# ---- FP6 (E3M2) path of the 4-bit layer ---------------------------------------------------------

def quik_fp6_row_bytes(K_b: int) -> int:
    return load().quik_fp6_row_bytes(K_b)


def quik_workspace_bytes_fp6(T: int, K: int, N: int, n_out: int) -> int:
    return load().quik_workspace_bytes_fp6(T, K, N, n_out)


def quik_weight_pack_fp6(w_q, K_b: int):
    """packed signed 4-bit weights uint8 [N, ldw] -> FP6 panels uint8 [stages, N, 48]."""
    w_q = _dev(w_q, torch.uint8, "w_q")
    N = w_q.shape[0]
    w6 = torch.empty((quik_fp6_row_bytes(K_b) // 48, N, 48), dtype=torch.uint8, device=w_q.device)
    rc = load().quik_weight_pack_fp6(_ptr(w_q), w_q.stride(0), N, K_b, _ptr(w6), _stream())
    _check(rc, "quik_weight_pack_fp6")
    return w6


def quik_quantize_fp6(x, outlier_idx, out=None):
    """x fp16 [T,K] -> (xq6 uint8 [stages,T,48], scale f32 [T], zero f32 [T], x_out f16 [T,n_out])."""
    x = _dev(x, torch.float16, "x")
    T, K = x.shape
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    if n_out:
        _dev(outlier_idx, torch.int32, "outlier_idx")
    ld6 = quik_fp6_row_bytes(K - n_out)
    if ld6 <= 0:
        raise QuikError(-1, "quik_fp6_row_bytes")
    if out is None:
        xq6 = torch.empty((ld6 // 48, T, 48), dtype=torch.uint8, device=x.device)
        scale = torch.empty(T, dtype=torch.float32, device=x.device)
        zero = torch.empty(T, dtype=torch.float32, device=x.device)
        x_out = torch.empty((T, n_out), dtype=torch.float16, device=x.device)
    else:
        xq6, scale, zero, x_out = out
    rc = load().quik_quantize_fp6(_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out,
                                  _ptr(xq6), _ptr(scale), _ptr(zero),
                                  _ptr(x_out) if n_out else None, x_out.stride(0) if n_out else 0, _stream())
    _check(rc, "quik_quantize_fp6")
    return xq6, scale, zero, x_out


def _gemm_dequant_fp6_args(xq6, scale, zero, x_out, K_b, w6, w_scale, w_reduced, w_out, bias, y):
    T, N = xq6.shape[1], w6.shape[1]
    n_out = 0 if x_out is None else int(x_out.shape[1])
    return (_ptr(xq6), _ptr(scale), _ptr(zero), _ptr(x_out) if n_out else None,
            x_out.stride(0) if n_out else 0, T, K_b, n_out, _ptr(w6), _ptr(w_scale), _ptr(w_reduced),
            _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0, _ptr(bias), N, _ptr(y), y.stride(0),
            _stream())


def quik_gemm_dequant_fp6(xq6, scale, zero, x_out, K_b: int, w6, w_scale, w_reduced, w_out, bias=None, out=None):
    xq6 = _dev(xq6, torch.uint8, "xq6")
    w6 = _dev(w6, torch.uint8, "w6")
    y = out if out is not None else torch.empty((xq6.shape[1], w6.shape[1]), dtype=torch.float16, device=xq6.device)
    rc = load().quik_gemm_dequant_fp6(*_gemm_dequant_fp6_args(xq6, scale, zero, x_out, K_b, w6, w_scale, w_reduced,
                                                              w_out, bias, y))
    _check(rc, "quik_gemm_dequant_fp6")
    return y


def prepare_gemm_dequant_fp6(xq6, scale, zero, x_out, K_b: int, w6, w_scale, w_reduced, w_out, bias, out):
    """Marshal-once form of quik_gemm_dequant_fp6 writing into `out`."""
    args = _gemm_dequant_fp6_args(xq6, scale, zero, x_out, K_b, w6, w_scale, w_reduced, w_out, bias, out)
    keep = (xq6, scale, zero, x_out, w6, w_scale, w_reduced, w_out, bias, out)
    return _prepared(load().quik_gemm_dequant_fp6, "quik_gemm_dequant_fp6", args, keep)


def prepare_quantize_fp6(x, outlier_idx, out):
    """Marshal-once form of quik_quantize_fp6 writing into out = (xq6, scale, zero, x_out)."""
    x = _dev(x, torch.float16, "x")
    T, K = x.shape
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    xq6, scale, zero, x_out = out
    args = (_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, _ptr(xq6),
            _ptr(scale), _ptr(zero), _ptr(x_out) if n_out else None, x_out.stride(0) if n_out else 0, _stream())
    return _prepared(load().quik_quantize_fp6, "quik_quantize_fp6", args, (x, outlier_idx, out))


def quik_int_gemm_fp6(xq6, w6, K_b: int):
    xq6 = _dev(xq6, torch.uint8, "xq6")
    w6 = _dev(w6, torch.uint8, "w6")
    T, N = xq6.shape[1], w6.shape[1]
    acc = torch.empty((T, N), dtype=torch.int32, device=xq6.device)
    rc = load().quik_int_gemm_fp6(_ptr(xq6), _ptr(w6), T, N, K_b, _ptr(acc), acc.stride(0), _stream())
    _check(rc, "quik_int_gemm_fp6")
    return acc


def _linear_fp6_args(x, outlier_idx, w6, w_scale, w_reduced, w_out, bias, y, workspace):
    T, K = x.shape
    N = w6.shape[1]
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    return (_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, _ptr(w6),
            _ptr(w_scale), _ptr(w_reduced), _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0,
            _ptr(bias), N, _ptr(y), y.stride(0), _ptr(workspace), workspace.numel(), _stream())


def _linear_fp6_buffers(x, outlier_idx, w6, out, workspace):
    x = _dev(x, torch.float16, "x")
    w6 = _dev(w6, torch.uint8, "w6")
    T, K = x.shape
    N = w6.shape[1]
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    need = quik_workspace_bytes_fp6(T, K, N, n_out)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=x.device)
    return y, workspace


def quik_linear_fp6(x, outlier_idx, w6, w_scale, w_reduced, w_out, bias=None, out=None, workspace=None):
    """Whole 4-bit layer on the FP6 matrix path.  Returns y fp16 [T, N]."""
    y, workspace = _linear_fp6_buffers(x, outlier_idx, w6, out, workspace)
    rc = load().quik_linear_fp6(*_linear_fp6_args(x, outlier_idx, w6, w_scale, w_reduced, w_out, bias, y, workspace))
    _check(rc, "quik_linear_fp6")
    return y


def prepare_linear_fp6(x, outlier_idx, w6, w_scale, w_reduced, w_out, bias=None, out=None, workspace=None):
    """Marshal-once form of quik_linear_fp6: returns (call, y)."""
    y, workspace = _linear_fp6_buffers(x, outlier_idx, w6, out, workspace)
    args = _linear_fp6_args(x, outlier_idx, w6, w_scale, w_reduced, w_out, bias, y, workspace)
    keep = (x, outlier_idx, w6, w_scale, w_reduced, w_out, bias, y, workspace)
    return _prepared(load().quik_linear_fp6, "quik_linear_fp6", args, keep), y


# ---- 2:4-sparse weights on the sparse int8 matrix instruction ------------------------------------

def quik_sp24_act_row_bytes(K_b: int) -> int:
    return load().quik_sp24_act_row_bytes(K_b)


def quik_sp24_weight_bytes(N: int, K_b: int) -> int:
    return load().quik_sp24_weight_bytes(N, K_b)


def quik_workspace_bytes_sp24(T: int, K: int, N: int, n_out: int) -> int:
    return load().quik_workspace_bytes_sp24(T, K, N, n_out)


def quik_weight_pack_sp24(w_q, K_b: int, check: bool = True):
    """packed signed 4-bit weights uint8 [N, ldw] -> uint8 [stages, N, 32].

    With check (the default) the call waits for the result and raises unless every group of four
    columns has at most two nonzero values."""
    w_q = _dev(w_q, torch.uint8, "w_q")
    N = w_q.shape[0]
    nbytes = quik_sp24_weight_bytes(N, K_b)
    if nbytes <= 0:
        raise QuikError(-1, "quik_sp24_weight_bytes")
    stages = quik_sp24_act_row_bytes(K_b) // 32
    w24 = torch.empty((stages, nbytes // (32 * stages), 32), dtype=torch.uint8, device=w_q.device)
    violations = torch.zeros(1, dtype=torch.int32, device=w_q.device) if check else None
    rc = load().quik_weight_pack_sp24(_ptr(w_q), w_q.stride(0), N, K_b, _ptr(w24), _ptr(violations), _stream())
    _check(rc, "quik_weight_pack_sp24")
    if check and int(violations.item()) != 0:
        raise QuikError(-1, "quik_weight_pack_sp24: %d groups of four with more than two nonzero weights"
                        % int(violations.item()))
    return w24


def quik_quantize_sp24(x, outlier_idx, out=None):
    """x fp16 [T,K] -> (xq24 uint8 [stages,T,32], scale f32 [T], zero f32 [T], x_out f16 [T,n_out])."""
    x = _dev(x, torch.float16, "x")
    T, K = x.shape
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    if n_out:
        _dev(outlier_idx, torch.int32, "outlier_idx")
    ld = quik_sp24_act_row_bytes(K - n_out)
    if ld <= 0:
        raise QuikError(-1, "quik_sp24_act_row_bytes")
    if out is None:
        xq24 = torch.empty((ld // 32, T, 32), dtype=torch.uint8, device=x.device)
        scale = torch.empty(T, dtype=torch.float32, device=x.device)
        zero = torch.empty(T, dtype=torch.float32, device=x.device)
        x_out = torch.empty((T, n_out), dtype=torch.float16, device=x.device)
    else:
        xq24, scale, zero, x_out = out
    rc = load().quik_quantize_sp24(_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out,
                                   _ptr(xq24), _ptr(scale), _ptr(zero),
                                   _ptr(x_out) if n_out else None, x_out.stride(0) if n_out else 0, _stream())
    _check(rc, "quik_quantize_sp24")
    return xq24, scale, zero, x_out


def _gemm_dequant_sp24_args(xq24, scale, zero, x_out, K_b, w24, w_scale, w_reduced, w_out, bias, y):
    T, N = xq24.shape[1], int(w_scale.numel())
    n_out = 0 if x_out is None else int(x_out.shape[1])
    return (_ptr(xq24), _ptr(scale), _ptr(zero), _ptr(x_out) if n_out else None,
            x_out.stride(0) if n_out else 0, T, K_b, n_out, _ptr(w24), _ptr(w_scale), _ptr(w_reduced),
            _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0, _ptr(bias), N, _ptr(y), y.stride(0),
            _stream())


def quik_gemm_dequant_sp24(xq24, scale, zero, x_out, K_b: int, w24, w_scale, w_reduced, w_out, bias=None, out=None):
    xq24 = _dev(xq24, torch.uint8, "xq24")
    w24 = _dev(w24, torch.uint8, "w24")
    y = out if out is not None else torch.empty((xq24.shape[1], int(w_scale.numel())), dtype=torch.float16,
                                                device=xq24.device)
    rc = load().quik_gemm_dequant_sp24(*_gemm_dequant_sp24_args(xq24, scale, zero, x_out, K_b, w24, w_scale,
                                                                w_reduced, w_out, bias, y))
    _check(rc, "quik_gemm_dequant_sp24")
    return y


def prepare_gemm_dequant_sp24(xq24, scale, zero, x_out, K_b: int, w24, w_scale, w_reduced, w_out, bias, out):
    """Marshal-once form of quik_gemm_dequant_sp24 writing into `out`."""
    args = _gemm_dequant_sp24_args(xq24, scale, zero, x_out, K_b, w24, w_scale, w_reduced, w_out, bias, out)
    keep = (xq24, scale, zero, x_out, w24, w_scale, w_reduced, w_out, bias, out)
    return _prepared(load().quik_gemm_dequant_sp24, "quik_gemm_dequant_sp24", args, keep)


def prepare_quantize_sp24(x, outlier_idx, out):
    """Marshal-once form of quik_quantize_sp24 writing into out = (xq24, scale, zero, x_out)."""
    x = _dev(x, torch.float16, "x")
    T, K = x.shape
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    xq24, scale, zero, x_out = out
    args = (_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, _ptr(xq24),
            _ptr(scale), _ptr(zero), _ptr(x_out) if n_out else None, x_out.stride(0) if n_out else 0, _stream())
    return _prepared(load().quik_quantize_sp24, "quik_quantize_sp24", args, (x, outlier_idx, out))


def quik_int_gemm_sp24(xq24, w24, N: int, K_b: int):
    xq24 = _dev(xq24, torch.uint8, "xq24")
    w24 = _dev(w24, torch.uint8, "w24")
    T = xq24.shape[1]
    acc = torch.empty((T, N), dtype=torch.int32, device=xq24.device)
    rc = load().quik_int_gemm_sp24(_ptr(xq24), _ptr(w24), T, N, K_b, _ptr(acc), acc.stride(0), _stream())
    _check(rc, "quik_int_gemm_sp24")
    return acc


def _linear_sp24_args(x, outlier_idx, w24, w_scale, w_reduced, w_out, bias, y, workspace):
    T, K = x.shape
    N = int(w_scale.numel())
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    return (_ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, _ptr(w24),
            _ptr(w_scale), _ptr(w_reduced), _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0,
            _ptr(bias), N, _ptr(y), y.stride(0), _ptr(workspace), workspace.numel(), _stream())


def _linear_sp24_buffers(x, outlier_idx, w24, w_scale, out, workspace):
    x = _dev(x, torch.float16, "x")
    w24 = _dev(w24, torch.uint8, "w24")
    T, K = x.shape
    N = int(w_scale.numel())
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    need = quik_workspace_bytes_sp24(T, K, N, n_out)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=x.device)
    return y, workspace


def quik_linear_sp24(x, outlier_idx, w24, w_scale, w_reduced, w_out, bias=None, out=None, workspace=None):
    """Whole 4-bit layer with 2:4-sparse weights.  Returns y fp16 [T, N]."""
    y, workspace = _linear_sp24_buffers(x, outlier_idx, w24, w_scale, out, workspace)
    rc = load().quik_linear_sp24(*_linear_sp24_args(x, outlier_idx, w24, w_scale, w_reduced, w_out, bias, y,
                                                    workspace))
    _check(rc, "quik_linear_sp24")
    return y


def prepare_linear_sp24(x, outlier_idx, w24, w_scale, w_reduced, w_out, bias=None, out=None, workspace=None):
    """Marshal-once form of quik_linear_sp24: returns (call, y)."""
    y, workspace = _linear_sp24_buffers(x, outlier_idx, w24, w_scale, out, workspace)
    args = _linear_sp24_args(x, outlier_idx, w24, w_scale, w_reduced, w_out, bias, y, workspace)
    keep = (x, outlier_idx, w24, w_scale, w_reduced, w_out, bias, y, workspace)
    return _prepared(load().quik_linear_sp24, "quik_linear_sp24", args, keep), y


def quik_ablation_workspace_bytes(T: int, K: int, N: int, n_out: int, bits: int) -> int:
    return load().quik_ablation_workspace_bytes(T, K, N, n_out, bits)


def quik_linear_ablation(version: int, x, outlier_idx, bits: int, w_q, w_scale, w_reduced,
                         w_out, bias=None, out=None, workspace=None):
    """The layer with unfused stages (version 1 or 2; 3 = quik_linear).  Returns (y, workspace)."""
    x = _dev(x, torch.float16, "x")
    w_q = _dev(w_q, torch.uint8, "w_q")
    T, K = x.shape
    N = w_q.shape[0]
    n_out = 0 if outlier_idx is None else int(outlier_idx.numel())
    need = quik_ablation_workspace_bytes(T, K, N, n_out, bits)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=x.device)
    rc = load().quik_linear_ablation(
        version, _ptr(x), T, K, x.stride(0), _ptr(outlier_idx) if n_out else None, n_out, bits,
        _ptr(w_q), w_q.stride(0), _ptr(w_scale), _ptr(w_reduced),
        _ptr(w_out) if n_out else None, w_out.stride(0) if n_out else 0, _ptr(bias), N, _ptr(y),
        y.stride(0), _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "quik_linear_ablation")
    return y, workspace


def workspace_views(workspace, T: int, K: int, N: int, n_out: int, bits: int):
    """Views (xq, scale, zero, x_out) into a workspace filled by quik_linear or quik_linear_ablation,
    at the places quik_workspace_regions reports."""
    off = (C.c_size_t * 4)()
    ldq = C.c_int(0)
    _check(load().quik_workspace_regions(T, K, N, n_out, bits, C.cast(off, C.c_void_p),
                                         C.cast(C.pointer(ldq), C.c_void_p)), "quik_workspace_regions")
    ldq = ldq.value
    xq = workspace[off[0]: off[0] + T * ldq].view(T, ldq)
    scale = workspace[off[1]: off[1] + T * 4].view(torch.float32)
    zero = workspace[off[2]: off[2] + T * 4].view(torch.float32)
    x_out = workspace[off[3]: off[3] + T * n_out * 2].view(torch.float16).view(T, n_out)
    return xq, scale, zero, x_out
