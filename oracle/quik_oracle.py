"""ctypes front end of the C oracle (oracle/quik_oracle.c).

TEST INFRASTRUCTURE ONLY: a slow, plain CPU implementation of "QUIK Matmul"
(Algorithm 1) used to check the GPU library.  Arrays are numpy, on the host.
fp16 tensors are passed as ``np.float16`` arrays and viewed as their bit
patterns; the C side has its own fp16 decoder.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

__all__ = [
    "OracleResult", "base_columns", "pack", "unpack", "quantize", "int_gemm", "weight_reduce",
    "fp_matmul", "dequant_add", "linear", "half_to_float", "num_threads",
]

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        for name in ("quik_oracle_base_columns", "quik_oracle_pack", "quik_oracle_unpack",
                     "quik_oracle_quantize", "quik_oracle_int_gemm", "quik_oracle_weight_reduce",
                     "quik_oracle_fp_matmul", "quik_oracle_dequant_add", "quik_oracle_linear"):
            getattr(_lib, name).restype = C.c_int
        _lib.quik_oracle_half_to_float.restype = None
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use on this host."""
    env = os.environ.get("OMP_NUM_THREADS")
    avail = len(os.sched_getaffinity(0))
    if env:
        try:
            return max(1, min(int(env.split(",")[0]), avail))
        except ValueError:
            pass
    return avail


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def _h(a, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float16:
        raise TypeError("expected float16")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def half_to_float(h: np.ndarray) -> np.ndarray:
    h = _h(h)
    out = np.empty(h.shape, np.float32)
    _load().quik_oracle_half_to_float(_p(h), C.c_int64(h.size), _p(out))
    return out


def base_columns(K: int, idx: np.ndarray) -> np.ndarray:
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    base = np.empty(K, np.int32)
    nb = _load().quik_oracle_base_columns(K, _p(idx), int(idx.size), _p(base))
    if nb < 0:
        raise ValueError(f"bad outlier index list (code {nb})")
    return base[:nb].copy()


def pack(q: np.ndarray, bits: int, activations: bool = False) -> np.ndarray:
    """Packed storage.  ``activations`` selects the activation nibble order (element 2p in the
    high nibble); the default is the weight order (element 2p in the low nibble)."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    rows, K_b = q.shape
    out = np.empty((rows, K_b * bits // 8), np.uint8)
    _chk(_load().quik_oracle_pack(_p(q), C.c_int64(rows), K_b, bits, int(activations), _p(out)), "pack")
    return out


def unpack(packed: np.ndarray, K_b: int, bits: int, activations: bool = False) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows = packed.shape[0]
    if packed.shape[1] != K_b * bits // 8:
        raise ValueError("packed row length does not match K_b and bits")
    out = np.empty((rows, K_b), np.int8)
    _chk(_load().quik_oracle_unpack(_p(packed), C.c_int64(rows), K_b, bits, int(activations), _p(out)),
         "unpack")
    return out


def quantize(x: np.ndarray, idx: np.ndarray, bits: int, audit: bool = False):
    """split + Quantization.  Returns (q int8 [T,K_b], scale f32 [T], zero f32 [T],
    x_out f16 [T,n_out]) and, with ``audit``, the tie-mismatch count as 5th item."""
    x = _h(x)
    T, K = x.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    n_out = int(idx.size)
    K_b = K - n_out
    q = np.empty((T, K_b), np.int8)
    scale = np.empty(T, np.float32)
    zero = np.empty(T, np.float32)
    x_out = np.empty((T, n_out), np.float16)
    mism = C.c_int64(0)
    rc = _load().quik_oracle_quantize(_p(x), T, K, _p(idx), n_out, bits, _p(q), _p(scale), _p(zero),
                                      _p(x_out), C.byref(mism) if audit else None)
    _chk(rc, "quantize")
    if audit:
        return q, scale, zero, x_out, int(mism.value)
    return q, scale, zero, x_out


def int_gemm(q: np.ndarray, wq: np.ndarray, bits: int) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    T, K_b = q.shape
    N = wq.shape[0]
    if wq.shape[1] != K_b:
        raise ValueError("K_b mismatch")
    acc = np.empty((T, N), np.int32)
    _chk(_load().quik_oracle_int_gemm(_p(q), _p(wq), T, N, K_b, bits, _p(acc)), "int_gemm")
    return acc


def weight_reduce(wq: np.ndarray, w_scale: np.ndarray) -> np.ndarray:
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    N, K_b = wq.shape
    w_scale = _h(w_scale, (N,))
    out = np.empty(N, np.float32)
    _chk(_load().quik_oracle_weight_reduce(_p(wq), _p(w_scale), N, K_b, _p(out)), "weight_reduce")
    return out


def fp_matmul(x_out: np.ndarray, w_out: np.ndarray) -> np.ndarray:
    x_out = _h(x_out)
    w_out = _h(w_out)
    T, n_out = x_out.shape
    N = w_out.shape[0]
    if w_out.shape[1] != n_out:
        raise ValueError("n_out mismatch")
    out = np.empty((T, N), np.float64)
    _chk(_load().quik_oracle_fp_matmul(_p(x_out), _p(w_out), T, N, n_out, _p(out)), "fp_matmul")
    return out


def dequant_add(acc, scale, zero, w_scale, w_reduced, result_fp, bits: int, bias=None) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    T, N = acc.shape
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    zero = np.ascontiguousarray(zero, dtype=np.float32)
    w_scale = _h(w_scale, (N,))
    w_reduced = np.ascontiguousarray(w_reduced, dtype=np.float32)
    if result_fp is not None:
        result_fp = np.ascontiguousarray(result_fp, dtype=np.float64)
        if result_fp.shape != (T, N):
            raise ValueError("result_fp shape")
    if bias is not None:
        bias = _h(bias, (N,))
    y = np.empty((T, N), np.float32)
    _chk(_load().quik_oracle_dequant_add(_p(acc), _p(scale), _p(zero), _p(w_scale), _p(w_reduced),
                                         _p(result_fp), _p(bias), T, N, bits, _p(y)), "dequant_add")
    return y


@dataclass
class OracleResult:
    y: np.ndarray          # float32 [T, N]
    q: np.ndarray          # int8 [T, K_b]
    scale: np.ndarray      # float32 [T]
    zero: np.ndarray       # float32 [T]
    x_out: np.ndarray      # float16 [T, n_out]
    acc: np.ndarray        # int32 [T, N]
    w_reduced: np.ndarray  # float32 [N]


def linear(x, idx, bits, w_packed, w_scale, w_out, bias=None, w_bits=None) -> OracleResult:
    """Whole layer (Algorithm 1, QUIK Matmul).  ``w_bits`` (default: ``bits``) is the width of the
    packed weights when it differs from the activations' (the W4A8 rows of the paper's precision
    ablation): the same steps of Algorithm 1, called one after the other with each operand's width."""
    if w_bits is not None and w_bits != bits:
        x = _h(x)
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        K_b = x.shape[1] - int(idx.size)
        wq = unpack(w_packed, K_b, w_bits)                         # weights: their own width
        w_reduced = weight_reduce(wq, w_scale)
        q, scale, zero, x_out = quantize(x, idx, bits)             # activations: theirs
        result_fp = fp_matmul(x_out, _h(w_out)) if idx.size else None
        acc = int_gemm(q, wq, max(bits, w_bits))                   # overflow bound of the wider operand
        y = dequant_add(acc, scale, zero, w_scale, w_reduced, result_fp, bits, bias=bias)   # halfRange of the activations
        return OracleResult(y, q, scale, zero, x_out, acc, w_reduced)
    x = _h(x)
    T, K = x.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    n_out = int(idx.size)
    K_b = K - n_out
    w_packed = np.ascontiguousarray(w_packed, dtype=np.uint8)
    N = w_packed.shape[0]
    if w_packed.shape[1] != K_b * bits // 8:
        raise ValueError("w_packed row length does not match K_b and bits")
    w_scale = _h(w_scale, (N,))
    w_out = _h(w_out, (N, n_out))
    if bias is not None:
        bias = _h(bias, (N,))
    r = OracleResult(np.empty((T, N), np.float32), np.empty((T, K_b), np.int8),
                     np.empty(T, np.float32), np.empty(T, np.float32),
                     np.empty((T, n_out), np.float16), np.empty((T, N), np.int32),
                     np.empty(N, np.float32))
    rc = _load().quik_oracle_linear(_p(x), T, K, _p(idx), n_out, bits, _p(w_packed), _p(w_scale),
                                    _p(w_out), _p(bias), N, _p(r.y), _p(r.q), _p(r.scale),
                                    _p(r.zero), _p(r.x_out), _p(r.acc), _p(r.w_reduced))
    _chk(rc, "linear")
    return r
