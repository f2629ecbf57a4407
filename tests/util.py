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


def e3m2_pattern(v: np.ndarray) -> np.ndarray:
    """Integers -8 .. 8 -> their bit patterns in the 6-bit float format E3M2 (1 sign bit, 3 exponent
    bits with bias 3, 2 mantissa bits), written from the format's definition:
    |v| = (1 + m/4) * 2^(e - 3) for e >= 1; zero is all-zero."""
    v = np.asarray(v, np.int64)
    mag = np.abs(v)
    out = np.zeros(v.shape, np.uint8)
    nz = mag > 0
    ex = np.zeros(v.shape, np.int64)
    ex[nz] = np.floor(np.log2(mag[nz])).astype(np.int64)
    frac4 = np.zeros(v.shape, np.int64)
    frac4[nz] = (mag[nz] * 4) // (1 << ex[nz]) - 4           # m: (|v| / 2^ex - 1) * 4
    assert np.all((mag[nz] * 4) % (1 << ex[nz]) == 0) and np.all(frac4 >= 0) and np.all(frac4 < 4)
    out[nz] = (((ex[nz] + 3) << 2) | frac4[nz]).astype(np.uint8)
    out[v < 0] |= 32
    return out


def fp6_panels(q: np.ndarray) -> np.ndarray:
    """Signed codes int [R, K_b] -> the byte image of "FP6 panels" as include/quik.h defines them,
    shaped [S, R, 48]: zero-padded to S stages of 64 columns; stage s of row r is block [s, r];
    a group of 32 columns is a 192-bit little-endian string (column j in bits [6j, 6j+6)); bytes
    0..15 of group g go to byte 16 g of the block, bytes 16..23 to byte 32 + 8 g."""
    R, K_b = q.shape
    S = (K_b + 63) // 64
    codes = np.zeros((R, 64 * S), np.uint8)
    codes[:, :K_b] = e3m2_pattern(q)
    bits = ((codes[:, :, None] >> np.arange(6, dtype=np.uint8)) & 1).astype(np.uint8)   # little-endian per code
    strings = np.packbits(bits.reshape(R, 2 * S, 192), axis=2, bitorder="little")       # [R, 2S, 24] bytes
    out = np.zeros((S, R, 48), np.uint8)
    for g in range(2):
        grp = strings[:, g::2, :]                      # [R, S, 24]: group g of every stage
        out[:, :, 16 * g: 16 * g + 16] = grp[:, :, :16].transpose(1, 0, 2)
        out[:, :, 32 + 8 * g: 40 + 8 * g] = grp[:, :, 16:].transpose(1, 0, 2)
    return out
