"""Heavy-hitter Q/K/V generator for the five benchmark workloads.

A *unit* is one (layer, sequence, head): units are independent in RoCo because
every attention head keeps its own cache and evicts at its own positions
(paper, Fig. 1 caption).  For each unit the generator draws

    Q, K, V ~ N(0, 1)  i.i.d.,  shape [T_total, d],  T_total = L + steps
    u       = a random unit vector (fixed per unit)
    K[heavy] += 4 u   at round(frac * T_total) distinct seeded positions
    Q        += 2 u   at every position

so that a small set of keys keeps receiving above-average attention from all
later queries (the attention-sink / heavy-hitter structure that attention-based
eviction policies rely on, paper section 4.1).  Rows [0, L) are the prompt,
rows [L, L+steps) are the per-step decode q / k_new / v_new with position
L + step.

Randomness is counter based: numpy's Philox keyed by (seed, config, layer,
sequence, head) with the tensor id placed in the high counter word, so any unit
can be regenerated alone, in any order, on any machine.

For bf16 workloads the draws are rounded to bf16 (round to nearest even) once,
here, and returned as float32 arrays whose values are exactly representable in
bf16: the HIP path stores them as bf16 without further rounding and the oracle
widens them to float64 without further rounding, so both consume identical
numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterator, List, Sequence, Tuple

import numpy as np

DEFAULT_SEED = 20240206


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); return float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = (bits + 0x7FFF + lsb) & 0xFFFF0000
    return rounded.astype(np.uint32).view(np.float32).reshape(x.shape)


@dataclass(frozen=True)
class WorkloadConfig:
    """Shape of one benchmark workload."""

    index: int
    name: str
    layers: int
    batch: int
    heads: int
    head_dim: int
    dtype: str  # "f32" or "bf16": storage type of Q/K/V and the cache
    prompt_len: int  # L
    budget: int  # B
    scope: int  # s: number of lowest-variance tokens inside the eviction scope
    steps: int  # decode steps after the prefill
    heavy_frac: Tuple[float, float] = (0.02, 0.02)  # first layer .. last layer
    recency_window: int = 0
    recency_bias: float = 0.0
    scope_sweep: Tuple[int, ...] = field(default_factory=tuple)

    @property
    def units(self) -> int:
        return self.layers * self.batch * self.heads

    @property
    def total_len(self) -> int:
        return self.prompt_len + self.steps

    def heavy_fraction(self, layer: int) -> float:
        lo, hi = self.heavy_frac
        if self.layers <= 1:
            return lo
        return lo + (hi - lo) * layer / (self.layers - 1)


CONFIGS: Tuple[WorkloadConfig, ...] = (
    WorkloadConfig(1, "tiny-fp32", 1, 1, 4, 64, "f32", 256, 128, 16, 64),
    WorkloadConfig(2, "7b-layer-prefill", 1, 1, 32, 128, "bf16", 4096, 2048, 128, 0),
    WorkloadConfig(3, "7b-layer-serving", 1, 16, 32, 128, "bf16", 3072, 2048, 64, 512),
    WorkloadConfig(4, "7b-32layer", 32, 8, 32, 128, "bf16", 8192, 1024, 32, 256,
                   heavy_frac=(0.005, 0.05)),
    WorkloadConfig(5, "13b-long-context", 1, 1, 40, 128, "bf16", 32768, 4096, 64, 1024,
                   recency_window=64, recency_bias=0.5,
                   scope_sweep=(16, 64, 256, 1024)),
)


@dataclass
class UnitInputs:
    """Inputs of one unit; float32 arrays (bf16-representable for bf16 configs)."""

    layer: int
    seq: int
    head: int
    Q: np.ndarray  # [T_total, d]
    K: np.ndarray
    V: np.ndarray
    heavy_positions: np.ndarray  # sorted int64 positions that received +4u


def _philox(seed: int, cfg_index: int, layer: int, seq: int, head: int,
            tensor_id: int) -> np.random.Generator:
    key0 = np.uint64(seed & 0xFFFFFFFFFFFFFFFF)
    key1 = np.uint64(((cfg_index & 0xFFFF) << 48) | ((layer & 0xFFFF) << 32)
                     | ((seq & 0xFFFF) << 16) | (head & 0xFFFF))
    counter = np.array([0, 0, 0, tensor_id], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=np.array([key0, key1], dtype=np.uint64),
                                                counter=counter))


def make_unit(cfg: WorkloadConfig, layer: int, seq: int, head: int,
              seed: int = DEFAULT_SEED, total_len: int | None = None) -> UnitInputs:
    """Generate Q, K, V of one unit.  `total_len` overrides L + steps (tests)."""
    T = cfg.total_len if total_len is None else int(total_len)
    d = cfg.head_dim
    g = lambda tid: _philox(seed, cfg.index, layer, seq, head, tid)  # noqa: E731
    Q = g(1).standard_normal((T, d), dtype=np.float32)
    K = g(2).standard_normal((T, d), dtype=np.float32)
    V = g(3).standard_normal((T, d), dtype=np.float32)
    u = g(4).standard_normal(d).astype(np.float64)
    u = (u / np.linalg.norm(u)).astype(np.float32)
    n_heavy = int(round(cfg.heavy_fraction(layer) * T))
    n_heavy = max(0, min(T, n_heavy))
    heavy = np.sort(g(5).choice(T, size=n_heavy, replace=False)) if n_heavy else \
        np.zeros(0, dtype=np.int64)
    K[heavy] += np.float32(4.0) * u
    Q += np.float32(2.0) * u
    if cfg.dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    return UnitInputs(layer, seq, head, Q, K, V, heavy.astype(np.int64))


def unit_ids(cfg: WorkloadConfig) -> List[Tuple[int, int, int]]:
    """(layer, seq, head) of every unit, in the flat unit order used everywhere."""
    return [(l, b, h) for l in range(cfg.layers) for b in range(cfg.batch)
            for h in range(cfg.heads)]


def make_units(cfg: WorkloadConfig, ids: Sequence[Tuple[int, int, int]] | None = None,
               seed: int = DEFAULT_SEED, total_len: int | None = None
               ) -> Iterator[UnitInputs]:
    """Yield the inputs of the given units (default: all of them, flat order)."""
    for (l, b, h) in (unit_ids(cfg) if ids is None else ids):
        yield make_unit(cfg, l, b, h, seed=seed, total_len=total_len)
