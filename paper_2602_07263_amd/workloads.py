"""Seeded synthetic workloads for the fused multi-LoRA linear layer.

This module only *draws inputs*: shapes, ranks, token segments, scales and random tensors with the
distributions the five benchmark configurations prescribe.  It holds none of the method's
arithmetic, imports neither the HIP binding nor the CPU oracle, and is the one piece both of
them are fed from (tests and the benchmark hand the same arrays to each side).

The synthetic tensors stand in for the paper's workload (Sec. 4.1: LoRA fine-tuning jobs of
rank 2..16 and batch 1..8 on 8B-class decoder models): only tensor shapes, segment structure
and value distributions reach this layer, so no dataset item or model weight is involved.

Conventions (all row-major):
  X  [T, d_in]   ~ N(0, 1)              dY [T, d_out] ~ N(0, 1)
  W  [d_in, d_out] ~ N(0, std 0.02)
  A_j [d_in, r_j] ~ U(-1/sqrt(d_in), +1/sqrt(d_in))   (Kaiming-uniform on fan-in d_in)
  B_j [r_j, d_out] ~ N(0, std 0.01)     (non-zero, so the adapter branch is exercised)
For bf16 workloads every tensor is rounded to bf16 (round-to-nearest-even) and returned as
float32 arrays whose values are exactly bf16-representable; both consumers see those values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np


@dataclass(frozen=True)
class Projection:
    name: str
    d_in: int
    d_out: int


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    dtype: str                      # "f32" or "bf16"
    projections: Sequence[Projection]
    ranks: Sequence[int]
    tokens: Sequence[int]           # tokens per job, in segment order
    scales: Sequence[float]

    @property
    def num_jobs(self) -> int:
        return len(self.ranks)

    @property
    def offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(np.asarray(self.tokens, dtype=np.int64))]).astype(np.int64)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.tokens))

    def flops(self, proj: Projection | None = None) -> float:
        """Algorithmic fwd+bwd flops: two base GEMMs plus six rank-GEMMs per job."""
        projs = [proj] if proj is not None else list(self.projections)
        tr = float(sum(t * r for t, r in zip(self.tokens, self.ranks)))
        T = float(self.total_tokens)
        return sum(4.0 * T * p.d_in * p.d_out + 6.0 * (p.d_in + p.d_out) * tr for p in projs)


@dataclass
class Problem:
    """One projection's tensors.  float32 numpy arrays (bf16-representable for bf16 workloads)."""
    dtype: str
    d_in: int
    d_out: int
    ranks: List[int]
    offsets: np.ndarray             # int64 [J+1]
    scales: List[float]
    X: np.ndarray
    W: np.ndarray
    dY: np.ndarray
    A: List[np.ndarray] = field(default_factory=list)
    B: List[np.ndarray] = field(default_factory=list)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def _cfg2_tokens() -> List[int]:
    # log-uniform draws in [256, 8192], snapped to multiples of 512 (minimum 512); the seed is the
    # first one whose total lands within 32768 +- 1024.
    rng = np.random.default_rng(9)
    u = np.exp(rng.uniform(np.log(256.0), np.log(8192.0), 8))
    return [int(v) for v in np.maximum(512, np.round(u / 512.0) * 512).astype(np.int64)]


def _cfg3_jobs():
    rng = np.random.default_rng(3)
    ranks = rng.choice([8, 16, 32, 64, 128], 16)
    batch = rng.integers(1, 5, 16)
    return [int(r) for r in ranks], [int(2048 * b) for b in batch]


def _cfg4_jobs():
    rng = np.random.default_rng(4)
    ranks = [int(r) for r in rng.choice([1, 3, 8, 48, 96, 256], 32)]
    draws = np.round(np.exp(rng.uniform(0.0, np.log(4096.0), 28))).astype(np.int64)
    tokens = np.concatenate([np.array([1, 17, 333, 16384], dtype=np.int64), draws])
    rng.shuffle(tokens)
    scales = [float(np.float32(s)) for s in rng.uniform(0.5, 4.0, 32)]
    return ranks, [int(t) for t in tokens], scales


def config(index: int) -> Workload:
    """The five benchmark configurations, 0-based."""
    if index == 0:
        return Workload("cfg0_tiny_f32", 0, "f32", [Projection("proj", 256, 256)], [4, 8], [64, 64], [2.0, 2.0])
    if index == 1:
        return Workload("cfg1_attn_proj_4096", 1, "bf16", [Projection("proj", 4096, 4096)],
                        [8, 16, 32, 64], [2048, 1024, 4096, 512], [2.0] * 4)
    if index == 2:
        return Workload("cfg2_mlp_8b", 2, "bf16",
                        [Projection("gate", 4096, 12288), Projection("up", 4096, 12288),
                         Projection("down", 12288, 4096)],
                        [4, 8, 8, 16, 32, 32, 64, 128], _cfg2_tokens(), [2.0] * 8)
    if index == 3:
        ranks, tokens = _cfg3_jobs()
        projs = [Projection("q", 4096, 4096), Projection("k", 4096, 1024), Projection("v", 4096, 1024),
                 Projection("o", 4096, 4096), Projection("gate", 4096, 12288), Projection("up", 4096, 12288),
                 Projection("down", 12288, 4096)]
        return Workload("cfg3_decoder_layer", 3, "bf16", projs, ranks, tokens, [2.0] * 16)
    if index == 4:
        ranks, tokens, scales = _cfg4_jobs()
        return Workload("cfg4_skew_14b_mlp", 4, "bf16",
                        [Projection("up", 5120, 17408), Projection("down", 17408, 5120)], ranks, tokens, scales)
    raise ValueError(f"no such config: {index}")


def custom(name: str, dtype: str, d_in: int, d_out: int, ranks, tokens, scales=None, index: int = 99) -> Workload:
    """An ad-hoc single-projection workload (edge-case tests)."""
    if scales is None:
        scales = [2.0] * len(ranks)
    return Workload(name, index, dtype, [Projection("proj", d_in, d_out)], list(ranks), list(tokens), list(scales))


def generate(wl: Workload, proj_index: int = 0, seed: int | None = None) -> Problem:
    """Draw one projection's tensors.  Draw order: W, X, dY, then (A_j, B_j) per job."""
    p = wl.projections[proj_index]
    rng = np.random.default_rng([wl.index if seed is None else seed, proj_index])
    T = wl.total_tokens
    W = rng.standard_normal((p.d_in, p.d_out), dtype=np.float32) * np.float32(0.02)
    X = rng.standard_normal((T, p.d_in), dtype=np.float32)
    dY = rng.standard_normal((T, p.d_out), dtype=np.float32)
    bound = 1.0 / np.sqrt(float(p.d_in))
    A, B = [], []
    for r in wl.ranks:
        A.append(rng.uniform(-bound, bound, (p.d_in, r)).astype(np.float32))
        B.append(rng.standard_normal((r, p.d_out), dtype=np.float32) * np.float32(0.01))
    if wl.dtype == "bf16":
        W, X, dY = round_to_bf16(W), round_to_bf16(X), round_to_bf16(dY)
        A = [round_to_bf16(a) for a in A]
        B = [round_to_bf16(b) for b in B]
    elif wl.dtype != "f32":
        raise ValueError(wl.dtype)
    return Problem(wl.dtype, p.d_in, p.d_out, list(wl.ranks), wl.offsets, [float(s) for s in wl.scales],
                   X, W, dY, A, B)
