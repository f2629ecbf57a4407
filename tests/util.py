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


def is_2of4(wq: np.ndarray) -> np.ndarray:
    """Per group of four consecutive columns: at most two nonzero values?  wq int [N, K_b], K_b % 4 == 0."""
    N, K_b = wq.shape
    return (wq.reshape(N, K_b // 4, 4) != 0).sum(axis=2) <= 2


def sp24_act_panels(q: np.ndarray) -> np.ndarray:
    """Signed codes int [T, K_b] -> the activation buffer of the 2:4-sparse path as include/quik.h
    defines it, shaped [S, T, 32]: zero-padded to S stages of 64 columns; byte 4 m + p of a stage's
    block holds column 8 m + p in the high nibble and column 8 m + 4 + p in the low nibble (two's
    complement)."""
    T, K_b = q.shape
    S = (K_b + 63) // 64
    nib = np.zeros((T, 64 * S), np.uint8)
    nib[:, :K_b] = q.astype(np.int64) & 0xF
    blk = nib.reshape(T, S, 8, 8)                       # [t, s, m, i]
    by = (blk[..., :4] << 4) | blk[..., 4:]             # [t, s, m, p]
    return np.ascontiguousarray(by.reshape(T, S, 32).transpose(1, 0, 2))


def sp24_weight_panels(wq: np.ndarray) -> np.ndarray:
    """Signed 4-bit weights int [N, K_b] -> the weight buffer of the 2:4-sparse path as include/quik.h
    defines it, shaped [S, N, 32] (per half: 8 bytes of values, the index word, 4 zero bytes).  Groups
    with more than two nonzero values keep their first two."""
    N, K_b = wq.shape
    S = (K_b + 63) // 64
    w = np.zeros((N, 64 * S), np.int64)
    w[:, :K_b] = wq
    grp = w.reshape(N, S, 16, 4)                        # [n, s, kappa, p]
    # kept positions: nonzero ones first, then the lowest unused, two in all, ascending
    key = np.where(grp != 0, 0, 4) + np.arange(4)
    keep = np.sort(np.argsort(key, axis=3, kind="stable")[..., :2], axis=3)      # [n, s, kappa, e]
    val = np.take_along_axis(grp, keep, axis=3) & 0xF
    out = np.zeros((S, N, 32), np.uint8)
    index = np.zeros((N, S, 2), np.uint64)
    for kappa in range(16):
        h, qq = (kappa // 4) % 2, 4 * (kappa // 8) + kappa % 4
        for e in range(2):
            c = 2 * qq + e
            byte = 16 * h + 4 * (c // 8) + c % 4
            shift = 0 if (c // 4) % 2 == 0 else 4
            out[:, :N, byte] |= (val[:, :, kappa, e].T << shift).astype(np.uint8)
            index[:, :, h] |= keep[:, :, kappa, e].astype(np.uint64) << np.uint64(2 * c)
    for h in range(2):
        word = index[:, :, h].T.astype(np.uint32)       # [s, n]
        for b in range(4):
            out[:, :N, 16 * h + 8 + b] = ((word >> (8 * b)) & 0xFF).astype(np.uint8)
    return out
