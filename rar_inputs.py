"""Seeded synthetic inputs for the all-reduce workloads (shared by oracle tests, GPU tests,
smoke and bench).  Holds none of the method's arithmetic: values come from numpy's
generators and the narrowing to bf16 is PyTorch's CPU cast, a library routine that neither
the oracle nor the HIP path uses.

The message shapes mirror the decode-phase tensor-parallel all-reduces of Section 5 of the
paper (batch x hidden bf16 activations, 128 KB - 2 MB) and the message-size sweep of its
micro-benchmark (Section 5, "Additional Setup Details"); the values are synthetic because a
collective's cost and schedule do not depend on them.

bf16 arrays are numpy uint16 bit patterns; fp32 arrays are numpy float32.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 20251109 * 1000


@dataclass(frozen=True)
class Workload:
    name: str
    index: int          # position in the configuration list, part of the seed
    P: int              # virtual ranks
    G: int              # ranks per node
    n: int              # elements per rank
    dtype: str          # "bf16" | "f32"
    values: str         # recipe name, see make_inputs

    @property
    def N(self) -> int:
        return self.P // self.G

    @property
    def bytes_per_rank(self) -> int:
        return self.n * (2 if self.dtype == "bf16" else 4)


WORKLOADS = {
    # P=8 (4 per node x 2 nodes), 128 KB bf16 per rank
    "c1": Workload("c1", 0, 8, 4, 65536, "bf16", "uniform"),
    "c1_int": Workload("c1_int", 0, 8, 4, 65536, "bf16", "ints"),
    # Llama-3.1-70B-shaped decode: hidden 8192 x 16 tokens, P=16
    "c2": Workload("c2", 1, 16, 4, 131072, "bf16", "normal_outliers"),
    # Llama-3.1-405B-shaped decode: hidden 16384 x 32 tokens, P=32
    "c3": Workload("c3", 2, 32, 4, 524288, "bf16", "normal"),
    # Llama-3.1-405B-shaped decode: hidden 16384 x 64 tokens, P=64
    "c4": Workload("c4", 3, 64, 4, 1048576, "bf16", "normal_rank_scale"),
}


def sweep_workload(P: int, G: int, bytes_per_rank: int, dtype: str) -> Workload:
    """One point of the message-size sweep (8 KB .. 64 MB per rank, N(0,1) values)."""
    es = 2 if dtype == "bf16" else 4
    return Workload(f"sweep_P{P}_G{G}_{bytes_per_rank}B_{dtype}", 4, P, G,
                    bytes_per_rank // es, dtype, "normal")


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> bf16 bit patterns (uint16) through torch's CPU cast."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> float32 (exact), for reporting only."""
    import torch
    t = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32)
    return t.numpy()


def _rank_values(rng: np.random.Generator, recipe: str, n: int) -> np.ndarray:
    if recipe == "uniform":
        return rng.uniform(-1.0, 1.0, n).astype(np.float32)
    if recipe == "ints":
        return rng.integers(-8, 9, n).astype(np.float32)
    if recipe == "normal":
        return rng.standard_normal(n, dtype=np.float32)
    if recipe == "normal_outliers":
        v = (0.5 * rng.standard_normal(n)).astype(np.float32)
        hit = rng.random(n) < 0.001
        sign = np.where(rng.random(n) < 0.5, -20.0, 20.0).astype(np.float32)
        return np.where(hit, sign, v)
    if recipe == "normal_rank_scale":
        scale = np.float32(rng.uniform(0.5, 2.0))
        return rng.standard_normal(n, dtype=np.float32) * scale
    raise ValueError(f"unknown recipe {recipe}")


def make_inputs(w: Workload, n: int | None = None) -> np.ndarray:
    """x[P, n] for workload w; each rank draws from its own seeded stream.
    n overrides the element count (used to cut a workload down for slow checks)."""
    n = w.n if n is None else n
    rows = []
    for p in range(w.P):
        rng = np.random.default_rng(SEED_BASE + 100 * w.index + p)
        rows.append(_rank_values(rng, w.values, n))
    x = np.stack(rows)
    return to_bf16_bits(x) if w.dtype == "bf16" else x.astype(np.float32)


def random_inputs(seed: int, P: int, n: int, dtype: str, recipe: str = "normal") -> np.ndarray:
    """Free-form seeded inputs for the edge-case tests."""
    rng = np.random.default_rng(seed)
    x = np.stack([_rank_values(rng, recipe, n) for _ in range(P)])
    return to_bf16_bits(x) if dtype == "bf16" else x.astype(np.float32)
