"""Seeded synthetic inputs for the QUIK linear layer.

This module only draws random tensors of the right shape, dtype and value
distribution.  It contains none of the method's arithmetic (no quantization, no
packing logic, no scale computation): the packed weight matrix is drawn directly
as uniformly random bytes, which is the same distribution as two independent
uniform signed nibbles per byte (or one uniform int8 for the 8-bit variant).

The same arrays are handed to the CPU oracle and to the HIP path by the tests,
the smoke check and the benchmark.  They stand in for the LLaMA-layer-shaped
benchmark of the paper (Section 4, layer-wise speedups): real activations and
weights are neither available nor needed to time or to check the layer.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20231009


@dataclass(frozen=True)
class LayerShape:
    """One synthetic workload: T tokens, K input features, N output features."""
    name: str
    T: int
    K: int
    N: int
    n_out: int
    bits: int = 4
    seed: int = BASE_SEED
    w_bits: int = 0          # weight bits when they differ from the activations' (0: same as bits)
    sparse24: bool = False   # 4-bit weights with two of every four consecutive base columns set to zero

    @property
    def K_b(self) -> int:
        return self.K - self.n_out

    @property
    def weight_bits(self) -> int:
        return self.w_bits or self.bits

    @property
    def row_bytes(self) -> int:
        """Bytes of one packed weight row of K_b quantized values."""
        return self.K_b * self.weight_bits // 8


# The five workload families named by the benchmark definition.  Index = config id.
CONFIGS = {
    "tiny": LayerShape("tiny", 16, 512, 512, 32, 4, BASE_SEED + 0),
    "llama7b_up": LayerShape("llama7b_up", 2048, 4096, 11008, 256, 4, BASE_SEED + 1),
    "llama7b_down": LayerShape("llama7b_down", 2048, 11008, 4096, 256, 4, BASE_SEED + 2),
    "llama7b_down_w8a8": LayerShape("llama7b_down_w8a8", 2048, 11008, 4096, 256, 8, BASE_SEED + 2),
    "llama7b_down_w4a8": LayerShape("llama7b_down_w4a8", 2048, 11008, 4096, 256, 8, BASE_SEED + 2, w_bits=4),
    "llama7b_down_w8a8_out896": LayerShape("llama7b_down_w8a8_out896", 2048, 11008, 4096, 896, 8, BASE_SEED + 2),
    "llama13b_qkv_t16": LayerShape("llama13b_qkv_t16", 16, 5120, 15360, 256, 4, BASE_SEED + 3),
    "llama13b_qkv_t128": LayerShape("llama13b_qkv_t128", 128, 5120, 15360, 256, 4, BASE_SEED + 3),
    "llama13b_qkv_t1024": LayerShape("llama13b_qkv_t1024", 1024, 5120, 15360, 256, 4, BASE_SEED + 3),
    "llama13b_qkv_t4096": LayerShape("llama13b_qkv_t4096", 4096, 5120, 15360, 256, 4, BASE_SEED + 3),
    "llama70b_up": LayerShape("llama70b_up", 4096, 8192, 28672, 256, 4, BASE_SEED + 4),
}


@dataclass
class LayerInputs:
    shape: LayerShape
    x: np.ndarray            # float16 [T, K]
    outlier_idx: np.ndarray  # int32 [n_out], sorted ascending, unique
    w_packed: np.ndarray     # uint8 [N, K_b*bits/8]; bits=4: two nibbles per byte
    w_scale: np.ndarray      # float16 [N]
    w_out: np.ndarray        # float16 [N, n_out]
    meta: dict = field(default_factory=dict)


def make_inputs(shape: LayerShape, outlier_gain: float = 40.0) -> LayerInputs:
    """Draw one layer's inputs.  Deterministic in ``shape.seed`` and the shape."""
    if (shape.K_b * shape.bits) % 8 != 0 or (shape.K_b * shape.weight_bits) % 8 != 0:
        raise ValueError("K_b * bits must be a multiple of 8")
    rng = np.random.Generator(np.random.PCG64(shape.seed))
    T, K, N, n_out = shape.T, shape.K, shape.N, shape.n_out
    idx = np.sort(rng.choice(K, size=n_out, replace=False)).astype(np.int32)
    x = rng.standard_normal((T, K), dtype=np.float32)
    if n_out:
        x[:, idx] *= np.float32(outlier_gain)
    x = x.astype(np.float16)
    w_packed = rng.integers(0, 256, size=(N, shape.row_bytes), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    w_out = (rng.standard_normal((N, n_out), dtype=np.float32) * np.float32(0.02)).astype(np.float16)
    if shape.sparse24:
        # 2:4 structure (Section 4.3.2 of the paper prunes with SparseGPT; here the two survivors of every
        # group of four nibbles = two bytes are drawn at random): AND with one of the six 16-bit masks
        # that keep two nibbles
        if shape.weight_bits != 4 or shape.K_b % 4:
            raise ValueError("sparse24 needs 4-bit weights and K_b a multiple of 4")
        keep = np.array([0x00FF, 0x0F0F, 0xF00F, 0x0FF0, 0xF0F0, 0xFF00], np.uint16)
        mask = keep[rng.integers(0, 6, size=(N, shape.row_bytes // 2))]
        w_packed = (w_packed.view(np.uint16) & mask).view(np.uint8)
    return LayerInputs(shape, x, idx, w_packed, w_scale, w_out)
