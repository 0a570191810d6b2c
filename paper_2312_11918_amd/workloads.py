"""Seeded synthetic Q/K/V inputs for the attention forward pass.

This module only draws random numbers and rounds them to 16-bit storage; it contains none of
the attention arithmetic and imports neither the GPU binding nor the CPU oracle, so both sides
can be fed the same bits.

The benchmark inputs of the paper (Section 7, "Results") are i.i.d. standard normal values;
the five workloads below keep that distribution at the shapes ``(B, H, N, d)`` listed in
``CONFIGS``.  Arrays are laid out ``[B, N, H, d]`` (Section 2: batch, seqlen, heads, headdim).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 20231211


@dataclass(frozen=True)
class Workload:
    index: int          # 1-based position in the list of workloads
    name: str
    B: int
    H: int
    N: int
    d: int
    dtype: str          # "fp16" or "bf16"
    k_outlier_frac: float = 0.0   # fraction of K rows (per head) multiplied by k_outlier_gain
    k_outlier_gain: float = 1.0

    @property
    def scale(self) -> float:
        """Softmax scale 1/sqrt(d) (Section 2), as the fp32 value handed to the kernel."""
        return float(np.float32(1.0) / np.sqrt(np.float32(self.d)))

    @property
    def flops(self) -> float:
        """FLOPs of the two matmuls only (Section 7): 4*B*H*N^2*d."""
        return 4.0 * self.B * self.H * float(self.N) ** 2 * self.d

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index


CONFIGS = {
    1: Workload(1, "tiny_B1_H2_N256_d64_fp16", 1, 2, 256, 64, "fp16"),
    2: Workload(2, "B32_H16_N512_d64_fp16", 32, 16, 512, 64, "fp16"),
    3: Workload(3, "B8_H16_N2048_d128_fp16", 8, 16, 2048, 128, "fp16"),
    4: Workload(4, "B2_H16_N8192_d128_bf16", 2, 16, 8192, 128, "bf16"),
    5: Workload(5, "B1_H32_N16384_d64_fp16_koutliers", 1, 32, 16384, 64, "fp16", 0.01, 8.0),
}


def round_to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values to 16-bit storage (round-to-nearest-even) and return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = x.view(np.uint32)
        lsb = (u >> np.uint32(16)) & np.uint32(1)
        return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_qkv(B: int, N: int, H: int, d: int, dtype: str, seed: int,
             k_outlier_frac: float = 0.0, k_outlier_gain: float = 1.0, Nk: int | None = None):
    """Draw Q, K, V ~ N(0,1) in that order from PCG64(seed) and round to ``dtype``.

    If ``k_outlier_frac`` > 0, then per (b, h) exactly ``round(frac*Nk)`` distinct key rows of K
    (drawn from the same generator, after V) are multiplied by ``k_outlier_gain`` before rounding.
    Returns three uint16 arrays of bit patterns: Q ``[B, N, H, d]``, K and V ``[B, Nk, H, d]``.
    """
    Nk = N if Nk is None else Nk
    rng = np.random.Generator(np.random.PCG64(seed))
    q = rng.standard_normal((B, N, H, d), dtype=np.float32)
    k = rng.standard_normal((B, Nk, H, d), dtype=np.float32)
    v = rng.standard_normal((B, Nk, H, d), dtype=np.float32)
    if k_outlier_frac > 0.0:
        n_out = int(round(k_outlier_frac * Nk))
        for b in range(B):
            for h in range(H):
                rows = rng.choice(Nk, size=n_out, replace=False)
                k[b, rows, h, :] *= np.float32(k_outlier_gain)
    return round_to_bits(q, dtype), round_to_bits(k, dtype), round_to_bits(v, dtype)


def make_workload(index: int):
    """The Q, K, V bit patterns of workload ``index`` (1..5) and its description."""
    w = CONFIGS[index]
    q, k, v = make_qkv(w.B, w.N, w.H, w.d, w.dtype, w.seed, w.k_outlier_frac, w.k_outlier_gain)
    return w, q, k, v
