"""GPU parity: the HIP library against the float64 oracle, element by element, through the C ABI."""
import math

import numpy as np
import pytest
import torch

from inputs import CONFIGS, make_unit, round_to_bf16
from oracle import roco_oracle as orc

pytestmark = pytest.mark.gpu


def _parity():
    import parity
    return parity


def run_workload(dtype, head_dim, units, lens, L_max, budget, scope, steps, seed, scale=0.0,
                 recency_window=0, recency_bias=0.0, want_out=True, cfg=None, tag=""):
    """Prefill-compress then `steps` lock-step decode steps on `units` synthetic units; returns tie counts."""
    P = _parity()
    cfg = cfg or CONFIGS[0 if dtype == "f32" else 1]
    sc = scale if scale > 0 else 1.0 / math.sqrt(head_dim)
    T = L_max + steps
    Q = np.zeros((units, T, head_dim), np.float32)
    K = np.zeros_like(Q)
    V = np.zeros_like(Q)
    rng = np.random.default_rng(seed)
    for u in range(units):
        # the workload generator at this test's own shape (head_dim / length differ from the config's)
        g = np.random.default_rng([seed, u])
        q, k, v = (g.standard_normal((T, head_dim), dtype=np.float32) for _ in range(3))
        d = g.standard_normal(head_dim)
        d = (d / np.linalg.norm(d)).astype(np.float32)
        heavy = g.choice(T, size=max(1, round(0.02 * T)), replace=False)
        k[heavy] += 4 * d
        q += 2 * d
        if dtype == "bf16":
            q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
        Q[u], K[u], V[u] = q, k, v
    sess = P.make_session(units, head_dim, budget, scope, dtype, scale, recency_window, recency_bias)
    print(f"[{tag}] prefill units={units} L_max={L_max} lens={list(lens)[:6]} B={budget} s={scope} {dtype} d={head_dim}", flush=True)
    g = P.gpu_prefill(sess, Q[:, :L_max].copy(), K[:, :L_max].copy(), V[:, :L_max].copy(), lens, want_out)
    ties = P.TieCount()
    states = []
    for u in range(units):
        res, t = P.check_prefill_unit(g, u, Q[u, :L_max], K[u, :L_max], V[u, :L_max], int(lens[u]), budget, scope,
                                      sc, dtype, recency_window, recency_bias, want_out)
        ties += t
        states.append(res.cache)
    next_pos = [int(l) for l in lens]
    for step in range(steps):
        t = L_max + step
        g_out, g_slot, g_pos = P.gpu_decode_step(sess, Q[:, t], K[:, t], V[:, t], next_pos)
        for u in range(units):
            ties += P.lockstep_decode_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t], K[u, t], V[u, t],
                                           next_pos[u], scope, sc, dtype, recency_window, recency_bias,
                                           what=f"[{tag}] step {step}")
            assert states[u].n_used <= budget
        next_pos = [p + 1 for p in next_pos]
        if step % 16 == 15 or step == steps - 1:
            host = P.cache_to_host(sess)
            for u in range(units):
                P.check_cache_unit(host, u, states[u], what=f"[{tag}] step {step}")
    print(f"[{tag}] ties: {ties}", flush=True)
    return ties


@pytest.mark.parametrize("seed", [20240206, 1, 2])
def test_config1_tiny_fp32_prefill_then_64_decode_steps(seed):
    """Workload 1 exactly: 4 heads x 64 dims fp32, 256 -> 128, scope 16, 64 steps, the config's own generator."""
    P = _parity()
    cfg = CONFIGS[0]
    L, B, s, d = cfg.prompt_len, cfg.budget, cfg.scope, cfg.head_dim
    units = [make_unit(cfg, 0, 0, h, seed=seed) for h in range(cfg.heads)]
    Q = np.stack([u.Q for u in units]); K = np.stack([u.K for u in units]); V = np.stack([u.V for u in units])
    sc = 1.0 / math.sqrt(d)
    sess = P.make_session(cfg.units, d, B, s, cfg.dtype)
    g = P.gpu_prefill(sess, Q[:, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), [L] * cfg.units, True)
    ties = P.TieCount()
    states = []
    for u in range(cfg.units):
        res, t = P.check_prefill_unit(g, u, Q[u, :L], K[u, :L], V[u, :L], L, B, s, sc, cfg.dtype)
        ties += t
        states.append(res.cache)
    for step in range(cfg.steps):
        t = L + step
        g_out, g_slot, g_pos = P.gpu_decode_step(sess, Q[:, t], K[:, t], V[:, t], [t] * cfg.units)
        for u in range(cfg.units):
            ties += P.lockstep_decode_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t], K[u, t], V[u, t], t, s, sc,
                                           cfg.dtype, what=f"cfg1 seed {seed} step {step}")
    host = P.cache_to_host(sess)
    for u in range(cfg.units):
        P.check_cache_unit(host, u, states[u], what=f"cfg1 seed {seed} end")
    print("cfg1 ties", ties, flush=True)
    assert ties.decode_decisions == cfg.units * cfg.steps and ties.prefill_decisions == cfg.units


@pytest.mark.parametrize("dtype,head_dim", [("bf16", 128), ("bf16", 64), ("f32", 128), ("f32", 64)])
def test_ragged_lengths_several_tiles_every_dtype(dtype, head_dim):
    """Lengths straddle the budget (some units never evict in prefill), ragged tails in every loop."""
    lens = [333, 97, 160, 161, 1, 300]
    run_workload(dtype, head_dim, len(lens), lens, 333, 160, 24, 20, seed=11, tag=f"ragged-{dtype}-{head_dim}")


def test_unit_that_fills_up_during_decode():
    """Cache below budget appends without evicting (evicted = -1) until it is full, then evicts."""
    lens = [10, 30, 37]
    run_workload("bf16", 128, 3, lens, 37, 40, 5, 36, seed=12, tag="fill-up")


@pytest.mark.parametrize("scope", [1, 7, 96])
def test_scope_extremes(scope):
    """scope = 1 (only the lowest-variance slot may go), scope = B (plain lowest mean attention score)."""
    run_workload("bf16", 128, 3, [200, 130, 96], 200, 96, scope, 12, seed=13, tag=f"scope-{scope}")


def test_budget_one_and_tiny_budgets():
    run_workload("f32", 64, 2, [9, 3], 9, 1, 1, 6, seed=14, tag="budget-1")
    run_workload("bf16", 128, 2, [50, 17], 50, 3, 2, 6, seed=15, tag="budget-3")


def test_recency_bias_prefill_and_decode():
    run_workload("bf16", 128, 3, [260, 200, 130], 260, 128, 16, 24, seed=16, recency_window=64, recency_bias=0.5,
                 tag="recency")


def test_explicit_scale():
    run_workload("f32", 64, 2, [150, 150], 150, 64, 8, 8, seed=17, scale=0.05, tag="scale")


def test_budget_not_smaller_than_everything_reproduces_full_attention():
    """B >= L + steps: nothing is ever evicted, outputs are plain causal attention."""
    run_workload("bf16", 128, 2, [70, 45], 70, 128, 9, 20, seed=18, tag="no-evict")


def test_larger_budget_many_splits_bf16():
    """B = 2048 at the serving shape's split configuration, a few units, short run."""
    run_workload("bf16", 128, 4, [2500, 2048, 2049, 2300], 2500, 2048, 64, 6, seed=19, want_out=False,
                 tag="b2048")


def test_exact_ties_go_to_the_lowest_index():
    """Duplicate tokens (identical k, and queries that cannot tell them apart) give bit-identical statistics
    on both sides only if accumulation orders agree, so this checks validity instead: with all-zero queries
    every probability is 1/(i+1), statistics depend on position only, and the variance / MAS orders are
    strict and known in closed form (test_oracle_pins: harmonic numbers)."""
    P = _parity()
    L, B, s, d = 96, 40, 6, 64
    Q = np.zeros((1, L, d), np.float32)
    rng = np.random.default_rng(5)
    K = rng.standard_normal((1, L, d)).astype(np.float32)
    V = rng.standard_normal((1, L, d)).astype(np.float32)
    sess = P.make_session(1, d, B, s, "f32")
    g = P.gpu_prefill(sess, Q, K, V, [L], True)
    res, ties = P.check_prefill_unit(g, 0, Q[0], K[0], V[0], L, B, s, 1 / math.sqrt(d), "f32")
    H = np.cumsum(1.0 / np.arange(1, L + 1))
    acc = H[-1] - np.concatenate([[0.0], H[:-1]])
    assert np.allclose(res.full.acc, acc, rtol=1e-12)


def test_budget_above_the_lds_key_limit_uses_the_workspace_keys():
    """B > 4096: the selection keeps its ranking keys in the workspace instead of LDS."""
    run_workload("bf16", 64, 1, [4300], 4300, 4100, 33, 5, seed=21, want_out=False, tag="b4100")


def test_select_victims_entry_point_reproduces_the_maintained_hint():
    """roco_select_victims on the current statistics gives the same next_slot the decode step keeps."""
    import paper_2402_06262_amd as roco
    P = _parity()
    rng = np.random.default_rng(3)
    units, L, B, s, d = 5, 150, 64, 9, 128
    Q = round_to_bf16(rng.standard_normal((units, L + 6, d)).astype(np.float32))
    K = round_to_bf16(rng.standard_normal((units, L + 6, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, L + 6, d)).astype(np.float32))
    lens = [150, 64, 63, 10, 100]
    sess = P.make_session(units, d, B, s, "bf16")
    P.gpu_prefill(sess, Q[:, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), lens, False)
    for step in range(6):
        c = sess.cache
        fresh = torch.full((units,), -5, dtype=torch.int32, device="cuda")
        roco.roco_select_victims(sess.params, c.stats, c.n_used, fresh, sess.decode_ws)
        torch.cuda.synchronize()
        full = (c.n_used == B).cpu().numpy()
        got, kept = fresh.cpu().numpy(), c.next_slot.cpu().numpy()
        assert np.array_equal(got[full], kept[full]), (step, got, kept)
        assert np.all(got[~full] == -1)
        # and the oracle agrees on the statistics the GPU holds (same fp32 values, widened)
        st = c.stats.cpu().numpy().astype(np.float64)
        for u in np.flatnonzero(full):
            mas = orc.mean_attention_score(st[u, 0], st[u, 2])
            var = np.maximum(0.0, (st[u, 1].astype(np.float32) / st[u, 2].astype(np.float32)
                                   - (st[u, 0].astype(np.float32) / st[u, 2].astype(np.float32)) ** 2).astype(np.float64))
            # fp32 keys, as the kernel ranks them; ties resolved by lowest slot on both sides
            mas32 = (st[u, 0].astype(np.float32) / st[u, 2].astype(np.float32)).astype(np.float64)
            assert orc.select_victim(mas32, var, s) == int(got[u])
        t = L + step
        P.gpu_decode_step(sess, Q[:, t], K[:, t], V[:, t], [l + step for l in lens])


@pytest.mark.parametrize("recency", [False, True])
def test_matrix_core_prefill_statistics_ragged_lengths(recency):
    """bf16 / head_dim 128 without the attention output runs the matrix-core kernels: lengths around every tile
    edge (32-row wave tiles, 64-row streamed tiles, 128-row workgroup tiles), with and without the recency bias."""
    lens = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 193, 300, 517]
    kw = dict(recency_window=64, recency_bias=0.5) if recency else {}
    run_workload("bf16", 128, len(lens), lens, 517, 100, 12, 3, seed=31, want_out=False, tag=f"mfma-ragged-{recency}", **kw)


def test_matrix_core_prefill_matches_vector_path_bitwise_decisions(monkeypatch):
    """Same inputs through the matrix-core kernels and through the vector-ALU kernels: retained sets agree and
    the statistics agree to fp32 rounding (the two paths differ only in summation order)."""
    P = _parity()
    rng = np.random.default_rng(41)
    units, L, B, s, d = 3, 700, 256, 32, 128
    Q = round_to_bf16(rng.standard_normal((units, L, d)).astype(np.float32) + 0.3)
    K = round_to_bf16(rng.standard_normal((units, L, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, L, d)).astype(np.float32))
    res = {}
    for mode in ("0", "1"):
        monkeypatch.setenv("ROCO_PREFILL_SIMPLE", mode)
        sess = P.make_session(units, d, B, s, "bf16")
        res[mode] = P.gpu_prefill(sess, Q, K, V, [700, 650, 300], False)
    assert np.array_equal(res["0"]["pos"], res["1"]["pos"])
    assert np.allclose(res["0"]["stats"], res["1"]["stats"], rtol=2e-5, atol=1e-9)
