"""The heavy-hitter generator of `heavy_hitter.py`, drawn on the GPU with torch's seeded generator.

For workloads too large to draw on the host in reasonable time (workload 4: 8192 units x 8448 tokens): the same
recipe -- Q, K, V ~ N(0, 1); a unit vector u per unit; K[heavy] += 4 u at exactly round(frac * T) distinct seeded
positions; Q += 2 u; one rounding to bf16 -- from another stream of random numbers (torch's Philox on the device
instead of numpy's on the host).  The library consumes the tensors where they are; the oracle gets host copies of
the units it checks, so both sides still see identical values.  No arithmetic of the method lives here.
"""
from __future__ import annotations

from typing import Tuple

from .heavy_hitter import DEFAULT_SEED, WorkloadConfig


def make_layer_on_device(cfg: WorkloadConfig, layer: int, seed: int = DEFAULT_SEED, total_len: int | None = None,
                         device: str = "cuda"):
    """Q, K, V of the batch x heads units of one layer, [units, T, d] in the workload's storage type on `device`
    (flat unit order: sequence-major, then head), and the heavy positions [units, n_heavy] (int64, unsorted)."""
    import torch

    T = cfg.total_len if total_len is None else int(total_len)
    U, d = cfg.batch * cfg.heads, cfg.head_dim
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + cfg.index * 1009 + layer) & 0x7FFFFFFFFFFFFFFF)
    Q = torch.randn((U, T, d), generator=g, device=device, dtype=torch.float32)
    K = torch.randn((U, T, d), generator=g, device=device, dtype=torch.float32)
    V = torch.randn((U, T, d), generator=g, device=device, dtype=torch.float32)
    u = torch.randn((U, d), generator=g, device=device, dtype=torch.float64)
    u = (u / u.norm(dim=1, keepdim=True)).float()
    n_heavy = max(0, min(T, int(round(cfg.heavy_fraction(layer) * T))))
    # distinct positions per unit: the n_heavy largest of T independent uniform keys
    heavy = torch.rand((U, T), generator=g, device=device).topk(n_heavy, dim=1).indices if n_heavy else \
        torch.zeros((U, 0), dtype=torch.int64, device=device)
    if n_heavy:
        rows = torch.arange(U, device=device)[:, None].expand(U, n_heavy)
        K[rows, heavy] += 4.0 * u[:, None, :]
    Q += 2.0 * u[:, None, :]
    if cfg.dtype == "bf16":
        Q, K, V = Q.to(torch.bfloat16), K.to(torch.bfloat16), V.to(torch.bfloat16)  # round to nearest even, once
    return Q, K, V, heavy
