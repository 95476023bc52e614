"""GPU parity on shapes drawn at random (seeded): the hand-picked cases elsewhere aim at known edges; this sweep aims
at the ones nobody thought of -- tile counts, ragged lengths, budgets, scopes, dtypes, recency windows, policies and
decode shapes in combinations that change which launch configuration the library picks."""
import numpy as np
import pytest

import test_gpu_parity as TP
import test_gpu_block as TB
import test_gpu_gqa as TG
from oracle import roco_oracle as orc

pytestmark = pytest.mark.gpu

POLICIES = [None, None, None, orc.Policy("aas", "all"), orc.Policy("mas", "window"), orc.Policy("oldest", "all", 3),
            orc.Policy("ltas", "window"), orc.Policy("aqas", "all")]


def draw(seed):
    r = np.random.default_rng([977, seed])
    dtype, d = [("bf16", 128), ("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)][r.integers(5)]
    units = int(r.integers(1, 6))
    L = int(r.integers(40, 900 if d == 128 and dtype == "bf16" else 400))
    B = int(r.integers(8, max(9, L)))
    lens = [int(x) for x in r.integers(max(1, L // 3), L + 1, size=units)]
    lens[int(r.integers(units))] = L
    pol = POLICIES[r.integers(len(POLICIES))]
    if pol is not None and pol.scope_kind == "window":
        s = max(1, B // 2)
    else:
        s = int(r.integers(1, B + 1))
    recency = bool(r.integers(3) == 0)
    steps = int(r.integers(3, 14))
    return dict(dtype=dtype, d=d, units=units, L=L, B=B, lens=lens, s=s, pol=pol, recency=recency, steps=steps)


@pytest.mark.parametrize("seed", range(48))
def test_prefill_and_decode_on_a_random_shape(seed, monkeypatch):
    c = draw(seed)
    monkeypatch.setenv("ROCO_DECODE_FUSED", str(seed % 2))  # both decode shapes over the sweep
    rw, rb = (int(5 + seed), 0.5) if c["recency"] else (0, 0.0)
    TP.run_workload(c["dtype"], c["d"], c["units"], c["lens"], c["L"], c["B"], c["s"], c["steps"], seed=3000 + seed,
                    recency_window=rw, recency_bias=rb, want_out=(seed % 3 == 0), tag=f"random-{seed}", policy=c["pol"])


@pytest.mark.parametrize("seed", range(16))
def test_grouped_prefill_and_steps_on_a_random_shape(seed):
    r = np.random.default_rng([978, seed])
    dtype, d = [("bf16", 128), ("f32", 64), ("bf16", 64)][r.integers(3)]
    group = int(r.integers(1, 6))
    units = int(r.integers(1, 4))
    L = int(r.integers(60, 500))
    B = 4 * int(r.integers(4, max(5, L // 4)))
    lens = [int(x) for x in r.integers(L // 2, L + 1, size=units)]
    lens[0] = L
    s = int(r.integers(1, B + 1))
    TG.run_grouped_prefill(dtype, d, group, lens, L, B, s, seed=4000 + seed, steps=int(r.integers(2, 7)),
                           recency=bool(r.integers(2)), tag=f"random-gqa-{seed}", want_out=bool(seed % 2))


@pytest.mark.parametrize("seed", range(16))
def test_block_steps_on_a_random_shape(seed):
    """Blocks of random sizes on caches of random fill (empty, partly filled, full), every dtype and head_dim."""
    r = np.random.default_rng([979, seed])
    dtype, d = [("bf16", 128), ("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)][r.integers(5)]
    units = int(r.integers(1, 4))
    B = 4 * int(r.integers(6, 80))
    s = int(r.integers(1, B + 1))
    if r.integers(3) == 0:
        prompt = [0] * units
    else:
        prompt = [int(x) for x in r.integers(1, 2 * B, size=units)]
    blocks = [int(x) for x in r.integers(1, 65 if seed % 2 else 33, size=int(r.integers(2, 7)))]  # one and two tiles of query rows
    blocks = [min(b, B) for b in blocks]
    TB.drive(units, d, B, s, prompt, blocks, seed=5000 + seed, recency=bool(r.integers(2)), tag=f"random-block-{seed}",
             dtype=dtype)


@pytest.mark.parametrize("seed", range(8))
def test_grouped_blocks_on_a_random_shape(seed):
    """Grouped-query blocks of random sizes, block x group up to 64 query rows, with and without the recency bias."""
    r = np.random.default_rng([980, seed])
    dtype, d = [("bf16", 128), ("bf16", 128), ("f32", 64), ("bf16", 64)][r.integers(4)]
    group = int([2, 3, 4, 5, 8, 16][r.integers(6)])
    units = int(r.integers(1, 4))
    B = 4 * int(r.integers(12, 60))
    s = int(r.integers(1, B + 1))
    cap = min(64 // group, B)
    blocks = [int(x) for x in r.integers(1, cap + 1, size=int(r.integers(4, 12)))] + [cap] * int(B // cap + 2)
    r.shuffle(blocks)
    TG.drive(units, B, s, group, blocks, seed=6000 + seed, recency=bool(r.integers(2)), tag=f"random-gqa-block-{seed}",
             dtype=dtype, d=d)
