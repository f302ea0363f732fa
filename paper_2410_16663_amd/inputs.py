"""Seeded synthetic inputs shared by the GPU path's callers and the oracle's callers.

Holds no attention arithmetic: only random draws, rounding to the 16-bit storage
formats, the five benchmark configurations and the row-sampling recipe.  Depends on
numpy alone and imports neither the GPU binding nor the oracle.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

F16 = 0
BF16 = 1


def f32_to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round fp32 values once (nearest-even) to fp16/bf16 and return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        u = x.view(np.uint32)
        bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        return ((u + bias) >> np.uint32(16)).astype(np.uint16)
    raise ValueError("dtype must be 0 (fp16) or 1 (bf16)")


def bits_to_f64(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Widen uint16 fp16/bf16 bit patterns exactly to fp64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError("dtype must be 0 (fp16) or 1 (bf16)")


@dataclass(frozen=True)
class Config:
    name: str
    index: int        # 1..5, fixes the seeds
    B: int
    H: int
    Nq: int
    Nk: int
    D: int
    dtype: int
    causal: bool
    mult: float = 1.0  # inputs are N(0,1) * mult
    window: int = 0    # > 0 (with causal): each row sees only the last `window` visible keys

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def seeds(self):
        return (1000 * self.index, 1000 * self.index + 1, 1000 * self.index + 2)

    def visible_pairs(self) -> int:
        """Number of (query, key) pairs that attend, per the mask."""
        if not self.causal:
            return self.B * self.H * self.Nq * self.Nk
        off = self.Nk - self.Nq
        i = np.arange(self.Nq, dtype=np.int64)
        n = np.clip(i + off + 1, 0, self.Nk)
        if self.window > 0:
            n = np.minimum(n, self.window)
        return int(self.B * self.H * n.sum())

    def flops(self) -> float:
        """4*B*H*Nq*Nk*D, halved when causal (the benchmark's FLOP convention)."""
        if self.window > 0:
            return 4.0 * self.D * self.visible_pairs()   # windowed: the exact count of attending pairs
        f = 4.0 * self.B * self.H * self.Nq * self.Nk * self.D
        return f / 2 if self.causal else f

    def describe(self) -> str:
        dt = "fp16" if self.dtype == F16 else "bf16"
        return (f"{self.name}: B={self.B} H={self.H} Nq={self.Nq} Nk={self.Nk} D={self.D} {dt} "
                f"{'causal' if self.causal else 'non-causal'}"
                + (f" window={self.window}" if self.window > 0 else "")
                + (f" inputs x{self.mult:g}" if self.mult != 1.0 else ""))


CONFIGS = {
    "C1": Config("C1", 1, 1, 2, 256, 256, 64, F16, True),
    "C2": Config("C2", 2, 1, 32, 2048, 2048, 128, F16, True),
    "C3": Config("C3", 3, 8, 32, 8192, 8192, 128, BF16, True),
    "C4": Config("C4", 4, 16, 16, 4096, 4096, 64, F16, False, 2.0),
    "C5": Config("C5", 5, 1, 32, 131072, 131072, 128, BF16, True),
}


# The decoding shape (appendix C of the paper: one new query per sequence against the cached keys
# and values) at a LLaMA-7B-like head layout, batch 2, 32768 cached tokens: the workload the
# split-KV entry point is measured on.  Not one of the five benchmark configurations.
DECODE = Config("DEC", 6, 2, 32, 1, 32768, 128, BF16, True)

# A causal sliding window (each token attends to the last 4096 tokens) over a 16384-token prefill at the
# same head layout: the workload the descriptor-mask entry point is measured on.  Not one of the five
# benchmark configurations either.
SLIDING = Config("SWA", 7, 2, 32, 16384, 16384, 128, BF16, True, 1.0, 4096)


# The same window at head dimension 64 (64 heads of 64 channels: the same hidden size), so that the descriptor-mask
# kernel is measured at both head dimensions.
SLIDING64 = Config("SWA64", 9, 2, 64, 16384, 16384, 64, BF16, True, 1.0, 4096)

# Chunked prefill: a chunk of 512 new tokens attends to a cache of 32768 tokens that ends with the chunk itself
# (bottom-right-aligned causal mask), one sequence at the same head layout.  512 rows are two query blocks per head,
# far too few workgroups to fill the chip, so this is the split-KV entry point's other shape (the first being the
# single-query decoding step).  Not one of the five benchmark configurations.
CHUNKED = Config("CHUNK", 10, 1, 32, 512, 32768, 128, BF16, True)

# Attention followed by the output projection, block of rows by block of rows (section 4.2): one sequence of
# 8192 tokens at the same head layout, a 4096 x 4096 projection matrix drawn as N(0,1)/sqrt(4096), blocks of 2048
# rows.  Not one of the five benchmark configurations.
PROJECTION = Config("LIN", 8, 1, 32, 8192, 8192, 128, BF16, True)
PROJECTION_N = 4096
PROJECTION_ROWS_PER_BLOCK = 2048


def normal_bits(shape, seed: int, dtype: int, mult: float = 1.0) -> np.ndarray:
    """i.i.d. N(0,1)*mult drawn in fp32 from PCG64(seed), rounded once to the storage format."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if mult != 1.0:
        x *= np.float32(mult)
    return f32_to_bits(x, dtype)


def make_qkv(cfg: Config):
    """Q, K, V bit patterns of a configuration, drawn in that order from its three seeds."""
    sq, sk, sv = cfg.seeds
    q = normal_bits((cfg.B, cfg.H, cfg.Nq, cfg.D), sq, cfg.dtype, cfg.mult)
    k = normal_bits((cfg.B, cfg.H, cfg.Nk, cfg.D), sk, cfg.dtype, cfg.mult)
    v = normal_bits((cfg.B, cfg.H, cfg.Nk, cfg.D), sv, cfg.dtype, cfg.mult)
    return q, k, v


def sample_rows(cfg: Config, per_head: int = 64, stratum: int = 128, seed: int | None = None) -> np.ndarray:
    """Seeded stratified sample of flat row ids (b*H+h)*Nq+i, ``per_head`` rows per (b,h).

    The Nq/stratum strata (blocks of ``stratum`` consecutive query rows) are dealt to the
    samples so that, over 16 consecutive heads, every stratum is hit when
    Nq/stratum <= 16*per_head: sample j of head index g takes stratum
    (16*j + g mod 16) mod nstrata, at a random offset inside it.  Row 0 and row Nq-1 of
    the first head are forced in.  Sorted per head, duplicates removed.
    """
    if seed is None:
        seed = 1000 * cfg.index + 999
    rng = np.random.Generator(np.random.PCG64(seed))
    nstrata = max(1, -(-cfg.Nq // stratum))
    out = []
    for g in range(cfg.B * cfg.H):
        j = np.arange(per_head, dtype=np.int64)
        s = (16 * j + (g % 16)) % nstrata
        r = rng.integers(0, stratum, size=per_head, dtype=np.int64)
        rows = np.minimum(s * stratum + r, cfg.Nq - 1)
        if g == 0:
            rows = np.concatenate([rows, np.array([0, cfg.Nq - 1], dtype=np.int64)])
        rows = np.unique(rows)
        out.append(g * cfg.Nq + rows)
    return np.concatenate(out)
