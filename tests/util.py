"""Shared helpers of the GPU parity tests (comparison rules, device upload)."""
from __future__ import annotations

import numpy as np


def to_dev(a, device="cuda"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def upload(inp):
    """Synthetic layer inputs -> device tensors in the layout the C ABI expects."""
    import torch
    d = {
        "x": to_dev(inp.x),
        "idx": to_dev(inp.outlier_idx) if inp.outlier_idx.size else None,
        "w_q": to_dev(inp.w_packed),
        "w_scale": to_dev(inp.w_scale),
        "w_out": to_dev(inp.w_out) if inp.outlier_idx.size else None,
    }
    # packed rows must start on 16-byte boundaries: pad the row stride if needed
    rb = inp.w_packed.shape[1]
    if rb % 16:
        ld = (rb + 15) // 16 * 16
        buf = torch.zeros((inp.w_packed.shape[0], ld), dtype=torch.uint8, device="cuda")
        buf[:, :rb] = d["w_q"]
        d["w_q"] = buf
    return d


def output_within_tolerance(y_gpu: np.ndarray, y_ref: np.ndarray, rel: float = 5e-3):
    """The fp16 output bar: |y - y_ref| <= rel * max(|y_ref|, 1e-3 * max|y_ref|) for
    every element, y_ref being the oracle's binary32 result."""
    y = y_gpu.astype(np.float64)
    r = y_ref.astype(np.float64)
    floor = 1e-3 * np.abs(r).max()
    tol = rel * np.maximum(np.abs(r), floor)
    err = np.abs(y - r)
    worst = float((err / tol).max()) if err.size else 0.0
    return bool(np.all(err <= tol)), worst


def expected_xq(oracle, q: np.ndarray, bits: int, ldq: int) -> np.ndarray:
    """Oracle codes -> the packed, zero-padded byte image the library must write."""
    packed = oracle.pack(q, bits, activations=True)
    out = np.zeros((q.shape[0], ldq), np.uint8)
    out[:, : packed.shape[1]] = packed
    return out
