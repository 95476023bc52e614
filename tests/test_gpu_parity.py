"""GPU parity: the HIP library against the float64 oracle, element by element, through the C ABI."""
import math

import numpy as np
import pytest
import torch

from inputs import CONFIGS, make_unit, round_to_bf16
from oracle import roco_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["split", "fused", "fused-streaming"])
def decode_path(request, monkeypatch):
    """Every case runs on both shapes of the decode step: slot ranges on several workgroups plus a finishing
    kernel, and one workgroup per unit doing the whole step (the library would pick by the number of units);
    the second also with the non-temporal K / V loads that caches beyond 192 MiB get."""
    monkeypatch.setenv("ROCO_DECODE_FUSED", "0" if request.param == "split" else "1")
    monkeypatch.setenv("ROCO_STREAMING_LOADS", "1" if request.param.endswith("streaming") else "0")
    return request.param


def _parity():
    import parity
    return parity


def run_workload(dtype, head_dim, units, lens, L_max, budget, scope, steps, seed, scale=0.0,
                 recency_window=0, recency_bias=0.0, want_out=True, cfg=None, tag="", policy=None):
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
    sess = P.make_session(units, head_dim, budget, scope, dtype, scale, recency_window, recency_bias, policy=policy)
    print(f"[{tag}] prefill units={units} L_max={L_max} lens={list(lens)[:6]} B={budget} s={scope} {dtype} d={head_dim}", flush=True)
    g = P.gpu_prefill(sess, Q[:, :L_max].copy(), K[:, :L_max].copy(), V[:, :L_max].copy(), lens, want_out)
    ties = P.TieCount()
    states = []
    for u in range(units):
        res, t = P.check_prefill_unit(g, u, Q[u, :L_max], K[u, :L_max], V[u, :L_max], int(lens[u]), budget, scope,
                                      sc, dtype, recency_window, recency_bias, want_out, policy=policy)
        ties += t
        states.append(res.cache)
    next_pos = [int(l) for l in lens]
    for step in range(steps):
        t = L_max + step
        g_out, g_slot, g_pos = P.gpu_decode_step(sess, Q[:, t], K[:, t], V[:, t], next_pos)
        for u in range(units):
            ties += P.lockstep_decode_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t], K[u, t], V[u, t],
                                           next_pos[u], scope, sc, dtype, recency_window, recency_bias,
                                           what=f"[{tag}] step {step}", policy=policy)
            assert states[u].n_used <= budget
        next_pos = [p + 1 for p in next_pos]
        if step % 16 == 15 or step == steps - 1:
            host = P.cache_to_host(sess)
            for u in range(units):
                P.check_cache_unit(host, u, states[u], what=f"[{tag}] step {step}")
    print(f"[{tag}] ties: {ties}", flush=True)
    P.assert_few_ties(ties, tag)
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
    P.assert_few_ties(ties, f"cfg1 seed {seed}", exact=True)


@pytest.mark.parametrize("dtype,head_dim", [("bf16", 128), ("bf16", 64), ("f32", 128), ("f32", 64)])
def test_ragged_lengths_several_tiles_every_dtype(dtype, head_dim):
    """Lengths straddle the budget (some units never evict in prefill), ragged tails in every loop."""
    lens = [333, 97, 160, 161, 1, 300]
    run_workload(dtype, head_dim, len(lens), lens, 333, 160, 24, 20, seed=11, tag=f"ragged-{dtype}-{head_dim}")


def test_unit_that_fills_up_during_decode():
    """Cache below budget appends without evicting (evicted = -1) until it is full, then evicts."""
    lens = [10, 30, 37]
    run_workload("bf16", 128, 3, lens, 37, 40, 5, 36, seed=12, tag="fill-up")


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_decode_from_an_empty_cache_without_any_prefill(dtype, d):
    """Token-wise generation from scratch: the first step attends the new token alone, nothing is evicted until the
    budget is reached, then every step evicts; the cache contents are compared at the end."""
    P = _parity()
    units, B, s, steps = 3, 24, 5, 40
    sc = 1.0 / math.sqrt(d)
    rng = np.random.default_rng(83)
    Q = rng.standard_normal((units, steps, d)).astype(np.float32) + 0.25
    K = rng.standard_normal((units, steps, d)).astype(np.float32)
    V = rng.standard_normal((units, steps, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    sess = P.make_session(units, d, B, s, dtype)
    states = [orc.CacheState(np.zeros((B, d)), np.zeros((B, d)), np.zeros(B), np.zeros(B), np.zeros(B),
                             np.full(B, -1, dtype=np.int64), 0) for _ in range(units)]
    ties = P.TieCount()
    for t in range(steps):
        g_out, g_slot, g_pos = P.gpu_decode_step(sess, Q[:, t], K[:, t], V[:, t], [t] * units)
        for u in range(units):
            ties += P.lockstep_decode_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t], K[u, t], V[u, t], t, s, sc,
                                           dtype, 0, 0.0, what=f"[from-empty] step {t}")
            assert states[u].n_used == min(t + 1, B)
            assert (int(g_slot[u]) >= 0) == (t >= B)
    host = P.cache_to_host(sess)
    for u in range(units):
        P.check_cache_unit(host, u, states[u], what="[from-empty] final cache")


def _poison_unused(cache, n_used):
    """Every byte of the cache slots (and statistics) at or beyond n_used[u] becomes 0xFF: NaN patterns in fp32 and in
    bf16.  The library must never let those bytes reach a result: such slots are documented as ignored."""
    for u, n in enumerate(n_used):
        cache.K[u, n:].view(torch.uint8).fill_(0xFF)
        cache.V[u, n:].view(torch.uint8).fill_(0xFF)
        cache.stats[u, :, n:].view(torch.uint8).fill_(0xFF)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_unused_cache_slots_may_hold_any_bytes_decode_from_empty(dtype, d):
    """Token-wise decode into a cache whose memory was never cleared: the first step's only row is the new token's,
    and the rows loaded merely to keep addresses in range (weight zero) must not turn the output into NaN."""
    P = _parity()
    units, B, s, steps = 3, 24, 5, 30
    sc = 1.0 / math.sqrt(d)
    rng = np.random.default_rng(84)
    Q = rng.standard_normal((units, steps, d)).astype(np.float32) + 0.25
    K = rng.standard_normal((units, steps, d)).astype(np.float32)
    V = rng.standard_normal((units, steps, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    sess = P.make_session(units, d, B, s, dtype)
    _poison_unused(sess.cache, [0] * units)
    states = [orc.CacheState(np.zeros((B, d)), np.zeros((B, d)), np.zeros(B), np.zeros(B), np.zeros(B),
                             np.full(B, -1, dtype=np.int64), 0) for _ in range(units)]
    for t in range(steps):
        g_out, g_slot, g_pos = P.gpu_decode_step(sess, Q[:, t], K[:, t], V[:, t], [t] * units)
        assert np.isfinite(g_out).all(), f"step {t}: bytes of an unused slot reached the output"
        for u in range(units):
            P.lockstep_decode_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t], K[u, t], V[u, t], t, s, sc, dtype, 0, 0.0,
                                   what=f"[poisoned-empty] step {t}")
    host = P.cache_to_host(sess)
    for u in range(units):
        P.check_cache_unit(host, u, states[u], what="[poisoned-empty] final cache")


def test_unused_cache_slots_may_hold_any_bytes_after_a_short_prompt():
    """A prompt that ends exactly where one workgroup's slot range ends (128 rows per range at this shape in the split
    decode step), budget above it: the next token's slot is the first row of the following range, whose bytes were
    never written.  Unused slots are poisoned after the prefill; the following steps must match the oracle."""
    P = _parity()
    units, L, B, s, d, steps = 3, 128, 512, 16, 128, 3
    lens = [128, 128, 256]
    rng = np.random.default_rng(85)
    T = 256 + steps
    Q = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32) + 0.25)
    K = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    sc = 1.0 / math.sqrt(d)
    sess = P.make_session(units, d, B, s, "bf16")
    g = P.gpu_prefill(sess, Q[:, :256].copy(), K[:, :256].copy(), V[:, :256].copy(), lens, False)
    states = [P.check_prefill_unit(g, u, Q[u, :256], K[u, :256], V[u, :256], lens[u], B, s, sc, "bf16", want_out=False)[0].cache
              for u in range(units)]
    _poison_unused(sess.cache, lens)
    pos = list(lens)
    for t in range(steps):
        g_out, g_slot, g_pos = P.gpu_decode_step(sess, Q[:, 256 + t], K[:, 256 + t], V[:, 256 + t], pos)
        assert np.isfinite(g_out).all(), f"step {t}: bytes of an unused slot reached the output"
        for u in range(units):
            P.lockstep_decode_unit(states[u], u, g_out, g_slot, g_pos, Q[u, 256 + t], K[u, 256 + t], V[u, 256 + t],
                                   pos[u], s, sc, "bf16", what=f"[poisoned-short-prompt] step {t}")
        pos = [p + 1 for p in pos]
    host = P.cache_to_host(sess)
    for u in range(units):
        n = states[u].n_used
        assert np.array_equal(host["stats"][u, 2][:n], states[u].count[:n])
        P.assert_stat_close(host["stats"][u, 0][:n], states[u].acc[:n], f"unit {u} Acc")
        P.assert_stat_close(host["stats"][u, 1][:n], states[u].acc2[:n], f"unit {u} Acc2")


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


def test_budgets_between_2048_and_the_lds_limit():
    """2048 < B <= 4096: the one-workgroup step loads part of the statistics after the stream, and keeps 12 bytes
    per slot in LDS; once with B a multiple of four (128-bit statistics accesses), once not (scalar accesses)."""
    run_workload("bf16", 128, 2, [3300, 3000], 3300, 3000, 50, 5, seed=23, want_out=False, tag="b3000")
    run_workload("f32", 64, 2, [2600, 2502], 2600, 2502, 40, 4, seed=24, want_out=False, tag="b2502")
    run_workload("bf16", 64, 1, [4200], 4200, 4096, 64, 3, seed=25, want_out=False, tag="b4096")


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


def test_budget_just_above_the_one_kernel_limit():
    """B > 4096 takes the split pair whatever the number of units; its ranking keys still fit the default LDS."""
    run_workload("bf16", 64, 1, [4300], 4300, 4100, 33, 5, seed=21, want_out=False, tag="b4100")


def test_budget_whose_ranking_keys_need_more_than_64_kib_of_lds():
    """8192 < B <= 16384: the selection kernels raise their dynamic LDS limit before the launch."""
    run_workload("bf16", 64, 1, [8300], 8300, 8200, 33, 4, seed=22, want_out=False, tag="b8200")


def test_budget_above_the_lds_key_limit_uses_the_workspace_keys():
    """B > 16384: the selection keeps its ranking keys in the workspace instead of LDS."""
    run_workload("bf16", 64, 1, [16500], 16500, 16400, 33, 3, seed=23, want_out=False, tag="b16400")


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
        roco.roco_select_victims(sess.params, c.stats, c.pos, c.n_used, fresh, sess.decode_ws)
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


@pytest.mark.parametrize("want_out", [False, True])
def test_matrix_core_prefill_scores_that_rise_far_above_the_earlier_ones(want_out):
    """The row passes keep a reference for their exponentials that is only raised when a tile's sum leaves the safe
    range: two keys deep inside the prompt whose scores lie 70-90 powers of two above everything before them (and
    the second as far above the first) force that path after the first tile, with and without the attention
    output; lengths end before, between and after the two keys."""
    P = _parity()
    units, L, B, s, d = 4, 700, 256, 24, 128
    lens = [700, 650, 300, 100]
    rng = np.random.default_rng(77)
    e = rng.standard_normal(d)
    e = (e / np.linalg.norm(e)).astype(np.float32)
    Q = rng.standard_normal((units, L, d)).astype(np.float32) + 8.0 * e
    K = rng.standard_normal((units, L, d)).astype(np.float32)
    V = rng.standard_normal((units, L, d)).astype(np.float32)
    K[:, 150] = 80.0 * e
    K[:, 420] = 160.0 * e
    Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    sess = P.make_session(units, d, B, s, "bf16")
    g = P.gpu_prefill(sess, Q, K, V, lens, want_out)
    for u in range(units):
        P.check_prefill_unit(g, u, Q[u], K[u], V[u], lens[u], B, s, 1.0 / math.sqrt(d), "bf16", 0, 0.0, want_out)


def test_matrix_core_prefill_with_one_block_per_workgroup(monkeypatch):
    """ROCO_PREFILL_PAIRED=0: every workgroup takes one block of rows instead of a long and a short one."""
    monkeypatch.setenv("ROCO_PREFILL_PAIRED", "0")
    run_workload("bf16", 128, 3, [700, 520, 300], 700, 256, 24, 0, seed=29, want_out=False, tag="unpaired")


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


def _small_serving_case(units=6, L=200, B=96, s=12, d=128, steps=8, seed=51):
    rng = np.random.default_rng(seed)
    T = L + steps
    Q = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32) + 0.2)
    K = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    return Q, K, V


def _state(c):
    return [t.clone() for t in (c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot)]


def _restore(c, st):
    for t, s in zip((c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot), st):
        t.copy_(s)


def test_results_are_bitwise_reproducible_run_to_run():
    """No float atomics, fixed combine order: two runs from scratch give identical bits."""
    P = _parity()
    Q, K, V = _small_serving_case()
    L, steps = 200, 8
    outs = []
    for _ in range(2):
        sess = P.make_session(6, 128, 96, 12, "bf16")
        P.gpu_prefill(sess, Q[:, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), [200, 180, 96, 97, 50, 200], True)
        rec = [sess.O.clone()]
        for t in range(steps):
            o, sl, ps = P.gpu_decode_step(sess, Q[:, L + t], K[:, L + t], V[:, L + t], [L + t] * 6)
            rec += [torch.from_numpy(o.copy()), torch.from_numpy(sl.copy())]
        rec += [x.cpu() for x in _state(sess.cache)]
        outs.append(rec)
    for a, b in zip(*outs):
        assert torch.equal(a.cpu(), b.cpu())


def test_decode_steps_captured_in_a_hip_graph_replay_like_eager_steps():
    """The decode step allocates nothing and never synchronises, so a caller can capture it.  Four steps are
    captured once and replayed three times, with eager work and synchronisations in between; every replay must
    leave exactly the state and outputs that the same steps leave when launched eagerly."""
    import paper_2402_06262_amd as roco
    P = _parity()
    units, L, B, s, d, steps = 6, 200, 96, 12, 128, 4
    Q, K, V = _small_serving_case(units, L, B, s, d, steps)
    sess = P.make_session(units, d, B, s, "bf16")
    P.gpu_prefill(sess, Q[:, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), [L] * units, False)
    c, p = sess.cache, sess.params
    dq = [P.to_dev(Q[:, L + t], "bf16") for t in range(steps)]
    dk = [P.to_dev(K[:, L + t], "bf16") for t in range(steps)]
    dv = [P.to_dev(V[:, L + t], "bf16") for t in range(steps)]
    qpos = [torch.full((units,), L + t, dtype=torch.int32, device="cuda") for t in range(steps)]
    out = [torch.zeros((units, d), dtype=torch.bfloat16, device="cuda") for _ in range(steps)]
    ev = [torch.zeros((units,), dtype=torch.int32, device="cuda") for _ in range(steps)]

    def run_steps():
        for t in range(steps):
            roco.roco_decode_step(p, dq[t], dk[t], dv[t], qpos[t], c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot,
                                  out[t], ev[t], None, sess.decode_ws)

    start = _state(c)
    # eager reference: three rounds of the same four steps (the state keeps evolving)
    want = []
    for _ in range(3):
        run_steps()
        torch.cuda.synchronize()
        want.append([x.clone() for x in out] + [x.clone() for x in ev] + _state(c))
    _restore(c, start)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up launch outside capture, as graph capture in torch asks for
        run_steps()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    _restore(c, start)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_steps()
    _restore(c, start)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device="cuda")
    for r in range(3):
        g.replay()
        scratch.add_(1.0)  # unrelated eager work between replays
        torch.cuda.synchronize()
        got = [x.clone() for x in out] + [x.clone() for x in ev] + _state(c)
        for a, b in zip(got, want[r]):
            assert torch.equal(a, b), f"replay {r} differs from the eager steps"
