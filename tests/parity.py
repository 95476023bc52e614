"""Parity harness: drive the HIP library and the CPU oracle on the same seeded inputs and compare.

Tolerances:
  * attention outputs: |g - o| <= tol * max(|o|, rms(o)) per vector, tol = 1e-3 (fp32 storage) or 2e-2
    (bf16 storage, whose rounding alone is 2^-9 relative);
  * Acc, Acc2:        |g - o| <= 1e-4 * max(|o|, 1e-6);  Count, pos, n_used, copied K/V rows: exact;
  * eviction decisions: identical index sets, unless the oracle's own gap lies inside the tie band
    (oracle/tie_band.py); such declared ties are counted, and the oracle adopts the library's choice so
    that later steps stay comparable.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
import torch

import paper_2402_06262_amd as roco
from oracle import roco_oracle as orc
from oracle import tie_band

STAT_RTOL = 1e-4  # fp32 sums of probabilities against float64: the worst of a full GPU run is 1.1e-5
STAT_FLOOR = 1e-6
OUT_RTOL = {"f32": 1e-3, "bf16": 2e-2}


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def roco_dtype(dtype: str) -> int:
    return roco.ROCO_BF16 if dtype == "bf16" else roco.ROCO_F32


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 host array (bf16-representable when dtype is bf16) -> device tensor of the storage type."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return t.to(torch_dtype(dtype)).contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.dtype in (torch.bfloat16, torch.float32) else t.detach().cpu().numpy()


# Run-wide records, printed at the end of a pytest session (tests/conftest.py): the worst output error in units of
# the tolerance under the floor in use (rms of the vector) and under the stricter floor 1e-3 * rms, per storage type;
# and every test's declared-tie count.
WORST_OUT = {"f32": [0.0, 0.0], "bf16": [0.0, 0.0]}
TIE_LOG: List[tuple] = []


def assert_out_close(g: np.ndarray, o: np.ndarray, dtype: str, what: str):
    g, o = np.asarray(g, np.float64), np.asarray(o, np.float64)
    rms = math.sqrt(float(np.mean(o * o))) if o.size else 0.0
    tol = OUT_RTOL[dtype] * np.maximum(np.abs(o), rms)
    if o.size:
        err = np.abs(g - o)
        w = WORST_OUT[dtype]
        w[0] = max(w[0], float(np.max(err / np.maximum(tol, 1e-300))))
        w[1] = max(w[1], float(np.max(err / np.maximum(OUT_RTOL[dtype] * np.maximum(np.abs(o), 1e-3 * rms), 1e-300))))
    bad = np.abs(g - o) > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} of {o.size} outside tolerance; worst |g-o|/tol = " \
                          f"{float(np.max(np.abs(g - o) / np.maximum(tol, 1e-300))):.3g}"


WORST_STAT = [0.0]  # largest |g - o| / max(|o|, STAT_FLOOR) of a run, printed at the end of a GPU run


def assert_stat_close(g: np.ndarray, o: np.ndarray, what: str):
    g, o = np.asarray(g, np.float64), np.asarray(o, np.float64)
    tol = STAT_RTOL * np.maximum(np.abs(o), STAT_FLOOR)
    if o.size:
        WORST_STAT[0] = max(WORST_STAT[0], float(np.max(np.abs(g - o) / np.maximum(np.abs(o), STAT_FLOOR))))
    bad = np.abs(g - o) > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} of {o.size} outside tolerance; worst rel = " \
                          f"{float(np.max(np.abs(g - o) / np.maximum(np.abs(o), STAT_FLOOR))):.3g}"


@dataclass
class TieCount:
    prefill_decisions: int = 0
    prefill_ties: int = 0
    decode_decisions: int = 0
    decode_ties: int = 0

    def __iadd__(self, o: "TieCount"):
        self.prefill_decisions += o.prefill_decisions
        self.prefill_ties += o.prefill_ties
        self.decode_decisions += o.decode_decisions
        self.decode_ties += o.decode_ties
        return self


def assert_few_ties(t: "TieCount", what: str, exact: bool = False):
    """Declared ties are decisions on which the library and the oracle differ inside the tolerance band; they must stay
    rare, or a wrong ranking could hide among them.  Ceiling: 1 % of the decisions (at least 2); `exact` (fp32 storage,
    where both sides rank nearly identical numbers): none at all."""
    dec, ties = t.prefill_decisions + t.decode_decisions, t.prefill_ties + t.decode_ties
    TIE_LOG.append((what, t.prefill_decisions, t.prefill_ties, t.decode_decisions, t.decode_ties))
    limit = 0 if exact else max(2, dec // 100)
    assert ties <= limit, f"{what}: {ties} declared ties in {dec} eviction decisions (limit {limit}): {t}"


@dataclass
class GpuSession:
    """Device buffers of one workload slice: `units` units with a common L_max and budget."""

    params: "roco.RocoParams"
    dtype: str
    cache: "roco.RocoCache"
    decode_ws: torch.Tensor
    out: torch.Tensor
    ev_slot: torch.Tensor
    ev_pos: torch.Tensor
    prefill_ws: Optional[torch.Tensor] = None
    O: Optional[torch.Tensor] = None


_IMPORTANCE = {"mas": 0, "aas": 1, "oldest": 2, "ltas": 3, "aqas": 4}

# The thresholded count (importance "aqas") adds 1 when p * n > 1.  A probability within AQAS_DELTA (relative) of the
# threshold can fall on either side in fp32 and in float64, so the two counts of a token may differ by the number of
# such near-threshold events it has seen.  The harness keeps that number per slot next to the oracle state
# (`state.slack`), compares the counts within it and uses it as the tie band of the eviction decision.
AQAS_DELTA = 1e-4


def _is_aqas(policy) -> bool:
    return policy is not None and policy.importance == "aqas"


def _near_threshold(p: np.ndarray, n_attended: int) -> np.ndarray:
    return (np.abs(np.asarray(p, dtype=np.float64) * n_attended - 1.0) <= AQAS_DELTA).astype(np.float64)


def assert_count_close(g: np.ndarray, o: np.ndarray, slack: np.ndarray, what: str):
    bad = np.abs(np.asarray(g, dtype=np.float64) - o) > slack
    assert not bad.any(), f"{what}: thresholded counts differ by more than the near-threshold events at {np.flatnonzero(bad)[:8]}"
_SCOPE_KIND = {"std": 0, "window": 1, "all": 2}


def make_session(units: int, head_dim: int, budget: int, scope: int, dtype: str, scale: float = 0.0,
                 recency_window: int = 0, recency_bias: float = 0.0, policy=None) -> GpuSession:
    """`policy`: an oracle Policy (None = RoCo); it is translated to the library's enum values here."""
    pol = policy or orc.ROCO
    p = roco.RocoParams(units, head_dim, budget, scope, roco_dtype(dtype), scale, recency_window, recency_bias,
                        _IMPORTANCE[pol.importance], _SCOPE_KIND[pol.scope_kind], pol.sinks)
    cache = roco.alloc_cache(p)
    ws = torch.empty(max(16, roco.decode_workspace_bytes(p)), dtype=torch.uint8, device="cuda")
    out = torch.zeros((units, head_dim), dtype=torch_dtype(dtype), device="cuda")
    ev_slot = torch.full((units,), -7, dtype=torch.int32, device="cuda")
    ev_pos = torch.full((units,), -7, dtype=torch.int32, device="cuda")
    return GpuSession(p, dtype, cache, ws, out, ev_slot, ev_pos)


def gpu_prefill(sess: GpuSession, Q: np.ndarray, K: np.ndarray, V: np.ndarray, lens: Sequence[int],
                want_out: bool = True):
    """Q, K, V: [units, L_max, d] float32 host arrays.  Returns host copies of everything written."""
    U, L_max, d = Q.shape
    p = sess.params
    assert U == p.units and d == p.head_dim
    dQ, dK, dV = to_dev(Q, sess.dtype), to_dev(K, sess.dtype), to_dev(V, sess.dtype)
    dlen = torch.tensor(list(lens), dtype=torch.int32, device="cuda")
    sess.prefill_ws = torch.empty(max(16, roco.prefill_workspace_bytes(p, L_max)), dtype=torch.uint8, device="cuda")
    sess.O = torch.zeros_like(dQ) if want_out else None
    c = sess.cache
    roco.roco_prefill_compress(p, dQ, dK, dV, dlen, L_max, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, sess.O, sess.prefill_ws)
    torch.cuda.synchronize()
    return dict(K=to_host(c.K), V=to_host(c.V), stats=to_host(c.stats), pos=to_host(c.pos),
                n_used=to_host(c.n_used), O=None if sess.O is None else to_host(sess.O))


def check_prefill_unit(g: dict, u: int, Qu, Ku, Vu, length: int, budget: int, scope: int, scale: float,
                       dtype: str, recency_window: int = 0, recency_bias: float = 0.0,
                       want_out: bool = True, row_block: int = 512, full=None, out_rows=None, policy=None):
    """Compare unit `u` of a gpu_prefill result with the oracle.  Returns (oracle result, TieCount).

    `full` lets several scopes share one evaluation of the oracle's statistics; `out_rows` restricts the
    comparison of the attention output to a sample of rows."""
    ties = TieCount()
    if full is None:
        full = orc.prefill_statistics(Qu, Ku, Vu, length, scale, recency_window, recency_bias, want_out, row_block,
                                      policy)
    res = orc.compress_from_statistics(full, Ku, Vu, length, budget, scope, policy=policy)
    n = min(length, budget)
    slack_full = None
    if _is_aqas(policy):  # near-threshold events of every prompt position, from the oracle's own rows
        slack_full = np.zeros(length)
        for i0, Prow in orc.causal_probability_rows(Qu, Ku, length, scale, recency_window, recency_bias, row_block):
            i1 = i0 + Prow.shape[0]
            causal = np.arange(i1)[None, :] <= np.arange(i0, i1)[:, None]
            near = np.abs(Prow * np.arange(i0 + 1, i1 + 1)[:, None] - 1.0) <= AQAS_DELTA
            slack_full[:i1] += (near & causal).sum(axis=0)
    assert int(g["n_used"][u]) == n, f"unit {u}: n_used {g['n_used'][u]} != {n}"
    gpos = g["pos"][u]
    assert np.all(gpos[n:] == -1), f"unit {u}: unused slots must have pos -1"
    assert np.all(np.diff(gpos[:n]) > 0), f"unit {u}: retained positions must ascend"
    assert gpos[:n].min() >= 0 and gpos[:n].max() < length
    if length > budget:
        ties.prefill_decisions += 1
        if not np.array_equal(gpos[:n], res.retained):
            mas, var, s_eff = orc.ranking_scores(policy, res.full.acc, res.full.acc2, res.full.count,
                                                 np.arange(length), scope)
            eps_m, eps_v = tie_band.bands_for(policy, res.full.acc, res.full.acc2, res.full.count)
            if slack_full is not None:
                eps_m = slack_full
            keep = np.zeros(length, bool)
            keep[gpos[:n]] = True
            ok, why = tie_band.admissible_eviction(mas, var, eps_m, eps_v, s_eff, length - budget,
                                                   np.flatnonzero(~keep))
            diff = sorted(set(gpos[:n].tolist()) ^ set(res.retained.tolist()))
            assert ok, f"unit {u}: retained set differs outside the tie band ({why}); differing positions {diff[:10]}"
            ties.prefill_ties += 1
            res = orc.compress_from_statistics(full, Ku, Vu, length, budget, scope, force_retained=gpos[:n],
                                               policy=policy)
    c = res.cache
    assert np.array_equal(gpos, c.pos)
    assert np.array_equal(g["stats"][u, 2], c.count), f"unit {u}: Count differs"
    assert_stat_close(g["stats"][u, 0], c.acc, f"unit {u} Acc")
    if slack_full is not None:
        c.slack = np.zeros(budget)
        c.slack[:n] = slack_full[c.pos[:n]]
        assert_count_close(g["stats"][u, 1], c.acc2, c.slack, f"unit {u} Acc2 (count)")
    else:
        assert_stat_close(g["stats"][u, 1], c.acc2, f"unit {u} Acc2")
    assert np.array_equal(g["K"][u, :n].astype(np.float64), c.K[:n]), f"unit {u}: cached K rows differ"
    assert np.array_equal(g["V"][u, :n].astype(np.float64), c.V[:n]), f"unit {u}: cached V rows differ"
    if want_out:
        for i in (range(length) if out_rows is None else out_rows):
            assert_out_close(g["O"][u, i], res.out[i], dtype, f"unit {u} O[{i}]")
    return res, ties


def gpu_decode_step(sess: GpuSession, q: np.ndarray, k: np.ndarray, v: np.ndarray, qpos: Sequence[int]):
    """q, k, v: [units, d] float32 host arrays.  Returns (out, evicted_slot, evicted_pos) on the host."""
    c, p = sess.cache, sess.params
    dq, dk, dv = to_dev(q, sess.dtype), to_dev(k, sess.dtype), to_dev(v, sess.dtype)
    dqpos = torch.tensor(list(qpos), dtype=torch.int32, device="cuda")
    roco.roco_decode_step(p, dq, dk, dv, dqpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, sess.out,
                          sess.ev_slot, sess.ev_pos, sess.decode_ws)
    torch.cuda.synchronize()
    return to_host(sess.out), to_host(sess.ev_slot), to_host(sess.ev_pos)


def lockstep_decode_unit(state: "orc.CacheState", u: int, g_out, g_slot, g_pos, q, k, v, qpos: int, scope: int,
                         scale: float, dtype: str, recency_window: int = 0, recency_bias: float = 0.0,
                         what: str = "", policy=None) -> TieCount:
    """Advance the oracle state of unit `u` by one step and compare with the library's step."""
    ties = TieCount()
    full = state.n_used == state.budget
    snapshot = state.copy() if full else None
    slack0 = getattr(state, "slack", np.zeros(state.budget)).copy() if _is_aqas(policy) else None
    r = orc.decode_step(state, q, k, v, qpos, scope, scale, recency_window, recency_bias, policy=policy)
    if full:
        ties.decode_decisions += 1
        if int(g_slot[u]) != r.evicted_slot:
            eps_m, eps_v = tie_band.bands_for(policy, snapshot.acc, snapshot.acc2, snapshot.count)
            if slack0 is not None:
                eps_m = slack0
            s_eff = state.budget if policy is not None and policy.scope_kind == "all" else scope
            ok, why = tie_band.admissible_eviction(r.mas, r.var, eps_m, eps_v, s_eff, 1, [int(g_slot[u])])
            assert ok, f"{what} unit {u}: victim slot {int(g_slot[u])} vs oracle {r.evicted_slot} outside the tie band ({why})"
            ties.decode_ties += 1
            # the oracle adopts the library's in-band choice: redo the step from the snapshot
            for name in ("K", "V", "acc", "acc2", "count", "pos"):
                getattr(state, name)[...] = getattr(snapshot, name)
            state.n_used = snapshot.n_used
            r = orc.decode_step(state, q, k, v, qpos, scope, scale, recency_window, recency_bias,
                                force_victim=int(g_slot[u]), policy=policy)
    assert int(g_slot[u]) == r.evicted_slot, f"{what} unit {u}: evicted_slot {int(g_slot[u])} != {r.evicted_slot}"
    assert int(g_pos[u]) == r.evicted_pos, f"{what} unit {u}: evicted_pos {int(g_pos[u])} != {r.evicted_pos}"
    assert_out_close(g_out[u], r.out, dtype, f"{what} unit {u} out")
    if slack0 is not None:
        n = state.n_used
        slack0[r.written_slot] = 0.0
        slack0[:n] += _near_threshold(r.probs, n)
        state.slack = slack0
    return ties


def check_cache_unit(sess_host: dict, u: int, state: "orc.CacheState", what: str = ""):
    n = state.n_used
    assert int(sess_host["n_used"][u]) == n, f"{what} unit {u}: n_used"
    assert np.array_equal(sess_host["pos"][u], state.pos), f"{what} unit {u}: pos"
    assert np.array_equal(sess_host["stats"][u, 2], state.count), f"{what} unit {u}: Count"
    assert_stat_close(sess_host["stats"][u, 0], state.acc, f"{what} unit {u} Acc")
    if hasattr(state, "slack"):
        assert_count_close(sess_host["stats"][u, 1], state.acc2, state.slack, f"{what} unit {u} Acc2 (count)")
    else:
        assert_stat_close(sess_host["stats"][u, 1], state.acc2, f"{what} unit {u} Acc2")
    assert np.array_equal(sess_host["K"][u, :n].astype(np.float64), state.K[:n]), f"{what} unit {u}: K rows"
    assert np.array_equal(sess_host["V"][u, :n].astype(np.float64), state.V[:n]), f"{what} unit {u}: V rows"


def cache_to_host(sess: GpuSession) -> dict:
    c = sess.cache
    return dict(K=to_host(c.K), V=to_host(c.V), stats=to_host(c.stats), pos=to_host(c.pos), n_used=to_host(c.n_used))


def gpu_encode_block(sess: GpuSession, block: int, q: np.ndarray, k: np.ndarray, v: np.ndarray, qpos0: Sequence[int],
                     ws: torch.Tensor):
    """q, k, v: [units, block, d] float32 host arrays.  Returns (out, evicted_slot, evicted_pos) on the host."""
    c, p = sess.cache, sess.params
    dq, dk, dv = to_dev(q, sess.dtype), to_dev(k, sess.dtype), to_dev(v, sess.dtype)
    dqpos = torch.tensor(list(qpos0), dtype=torch.int32, device="cuda")
    out = torch.zeros((p.units, block, p.head_dim), dtype=torch_dtype(sess.dtype), device="cuda")
    es = torch.full((p.units, block), -7, dtype=torch.int32, device="cuda")
    ep = torch.full((p.units, block), -7, dtype=torch.int32, device="cuda")
    roco.roco_encode_block(p, block, dq, dk, dv, dqpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, out, es, ep, ws)
    torch.cuda.synchronize()
    return to_host(out), to_host(es), to_host(ep)


def lockstep_block_unit(state: "orc.CacheState", u: int, g_out, g_slot, g_pos, q, k, v, qpos0: int, scope: int,
                        scale: float, dtype: str, recency_window: int = 0, recency_bias: float = 0.0,
                        what: str = "", policy=None) -> TieCount:
    """Advance the oracle state of unit `u` by one block and compare with the library's block step."""
    ties = TieCount()
    b = q.shape[0]
    n = state.n_used
    E = max(0, n + b - state.budget)
    snapshot = state.copy()
    slack0 = getattr(state, "slack", np.zeros(state.budget)).copy() if _is_aqas(policy) else None
    r = orc.encode_block(state, q, k, v, qpos0, scope, scale, recency_window, recency_bias, policy=policy)
    g_ev = sorted(int(x) for x in g_slot[u] if x >= 0)
    if E > 0:
        ties.decode_decisions += 1
        if g_ev != sorted(int(x) for x in r.evicted_slot if x >= 0):
            eps_m, eps_v = tie_band.bands_for(policy, snapshot.acc[:n], snapshot.acc2[:n], snapshot.count[:n])
            if slack0 is not None:
                eps_m = slack0[:n]
            s_eff = n if policy is not None and policy.scope_kind == "all" else scope
            ok, why = tie_band.admissible_eviction(r.mas, r.var, eps_m, eps_v, s_eff, E, g_ev)
            assert ok, f"{what} unit {u}: evicted slots {g_ev} outside the tie band ({why})"
            ties.decode_ties += 1
            for name in ("K", "V", "acc", "acc2", "count", "pos"):
                getattr(state, name)[...] = getattr(snapshot, name)
            state.n_used = snapshot.n_used
            r = orc.encode_block(state, q, k, v, qpos0, scope, scale, recency_window, recency_bias,
                                 force_evicted=np.array(g_ev), policy=policy)
    assert np.array_equal(g_slot[u], r.evicted_slot), f"{what} unit {u}: evicted_slot {g_slot[u]} != {r.evicted_slot}"
    assert np.array_equal(g_pos[u], r.evicted_pos), f"{what} unit {u}: evicted_pos {g_pos[u]} != {r.evicted_pos}"
    for i in range(b):
        assert_out_close(g_out[u, i], r.out[i], dtype, f"{what} unit {u} out[{i}]")
    if slack0 is not None:
        slack0[r.slots] = 0.0
        n_new = state.n_used
        for i in range(b):
            seen = r.probs[i] > 0.0  # the slots row i attended (a probability is never exactly zero)
            slack0[:n_new] += np.where(seen, _near_threshold(r.probs[i], int(seen.sum())), 0.0)
        state.slack = slack0
    return ties


def gpu_decode_step_gqa(sess: GpuSession, group: int, q: np.ndarray, k: np.ndarray, v: np.ndarray,
                        qpos: Sequence[int], ws: torch.Tensor):
    """q: [units, group, d], k, v: [units, d] float32 host arrays.  Returns (out, evicted_slot, evicted_pos)."""
    c, p = sess.cache, sess.params
    dq, dk, dv = to_dev(q, sess.dtype), to_dev(k, sess.dtype), to_dev(v, sess.dtype)
    dqpos = torch.tensor(list(qpos), dtype=torch.int32, device="cuda")
    out = torch.zeros((p.units, group, p.head_dim), dtype=torch_dtype(sess.dtype), device="cuda")
    es = torch.full((p.units,), -7, dtype=torch.int32, device="cuda")
    ep = torch.full((p.units,), -7, dtype=torch.int32, device="cuda")
    roco.roco_decode_step_gqa(p, group, dq, dk, dv, dqpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, out, es,
                              ep, ws)
    torch.cuda.synchronize()
    return to_host(out), to_host(es), to_host(ep)


def lockstep_gqa_unit(state: "orc.CacheState", u: int, g_out, g_slot, g_pos, Qg, k, v, qpos: int, scope: int,
                      scale: float, dtype: str, recency_window: int = 0, recency_bias: float = 0.0,
                      what: str = "") -> TieCount:
    """Advance the oracle state of key/value head `u` by one grouped-query step and compare with the library's."""
    ties = TieCount()
    full = state.n_used == state.budget
    snapshot = state.copy() if full else None
    r = orc.decode_step_gqa(state, Qg, k, v, qpos, scope, scale, recency_window, recency_bias)
    if full:
        ties.decode_decisions += 1
        if int(g_slot[u]) != r.evicted_slot:
            eps_m, eps_v = tie_band.bands(snapshot.acc, snapshot.acc2, snapshot.count)
            ok, why = tie_band.admissible_eviction(r.mas, r.var, eps_m, eps_v, scope, 1, [int(g_slot[u])])
            assert ok, f"{what} unit {u}: victim slot {int(g_slot[u])} vs oracle {r.evicted_slot} outside the tie band ({why})"
            ties.decode_ties += 1
            for name in ("K", "V", "acc", "acc2", "count", "pos"):
                getattr(state, name)[...] = getattr(snapshot, name)
            state.n_used = snapshot.n_used
            r = orc.decode_step_gqa(state, Qg, k, v, qpos, scope, scale, recency_window, recency_bias,
                                    force_victim=int(g_slot[u]))
    assert int(g_slot[u]) == r.evicted_slot, f"{what} unit {u}: evicted_slot {int(g_slot[u])} != {r.evicted_slot}"
    assert int(g_pos[u]) == r.evicted_pos, f"{what} unit {u}: evicted_pos {int(g_pos[u])} != {r.evicted_pos}"
    for h in range(Qg.shape[0]):
        assert_out_close(g_out[u, h], r.out[h], dtype, f"{what} unit {u} head {h} out")
    return ties


def gpu_encode_block_gqa(sess: GpuSession, block: int, group: int, q: np.ndarray, k: np.ndarray, v: np.ndarray,
                         qpos0: Sequence[int], ws: torch.Tensor):
    """q: [units, block, group, d], k, v: [units, block, d] float32 host arrays."""
    c, p = sess.cache, sess.params
    dq, dk, dv = to_dev(q, sess.dtype), to_dev(k, sess.dtype), to_dev(v, sess.dtype)
    dqpos = torch.tensor(list(qpos0), dtype=torch.int32, device="cuda")
    out = torch.zeros((p.units, block, group, p.head_dim), dtype=torch_dtype(sess.dtype), device="cuda")
    es = torch.full((p.units, block), -7, dtype=torch.int32, device="cuda")
    ep = torch.full((p.units, block), -7, dtype=torch.int32, device="cuda")
    roco.roco_encode_block_gqa(p, block, group, dq, dk, dv, dqpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, out,
                               es, ep, ws)
    torch.cuda.synchronize()
    return to_host(out), to_host(es), to_host(ep)


def lockstep_block_gqa_unit(state: "orc.CacheState", u: int, g_out, g_slot, g_pos, q, k, v, qpos0: int, scope: int,
                            scale: float, dtype: str, recency_window: int = 0, recency_bias: float = 0.0,
                            what: str = "") -> TieCount:
    """Advance the oracle state of key/value head `u` by one grouped block (q: [b, g, d]) and compare."""
    ties = TieCount()
    b, g = q.shape[0], q.shape[1]
    n = state.n_used
    E = max(0, n + b - state.budget)
    snapshot = state.copy()
    r = orc.encode_block_gqa(state, q, k, v, qpos0, scope, scale, recency_window, recency_bias)
    g_ev = sorted(int(x) for x in g_slot[u] if x >= 0)
    if E > 0:
        ties.decode_decisions += 1
        if g_ev != sorted(int(x) for x in r.evicted_slot if x >= 0):
            eps_m, eps_v = tie_band.bands(snapshot.acc[:n], snapshot.acc2[:n], snapshot.count[:n])
            ok, why = tie_band.admissible_eviction(r.mas, r.var, eps_m, eps_v, scope, E, g_ev)
            assert ok, f"{what} unit {u}: evicted slots {g_ev} outside the tie band ({why})"
            ties.decode_ties += 1
            for name in ("K", "V", "acc", "acc2", "count", "pos"):
                getattr(state, name)[...] = getattr(snapshot, name)
            state.n_used = snapshot.n_used
            r = orc.encode_block_gqa(state, q, k, v, qpos0, scope, scale, recency_window, recency_bias,
                                     force_evicted=np.array(g_ev, dtype=np.int64))
    assert np.array_equal(g_slot[u], r.evicted_slot), f"{what} unit {u}: evicted_slot {g_slot[u]} != {r.evicted_slot}"
    assert np.array_equal(g_pos[u], r.evicted_pos), f"{what} unit {u}: evicted_pos {g_pos[u]} != {r.evicted_pos}"
    for i in range(b):
        for h in range(g):
            assert_out_close(g_out[u, i, h], r.out[i, h], dtype, f"{what} unit {u} token {i} head {h} out")
    return ties


def gpu_prefill_gqa(sess: GpuSession, group: int, Q: np.ndarray, K: np.ndarray, V: np.ndarray, lens: Sequence[int],
                    want_out: bool = False):
    """Q: [units, group, L_max, d]; K, V: [units, L_max, d] float32 host arrays.  Host copies of what was written."""
    U, g, L_max, d = Q.shape
    p = sess.params
    assert U == p.units and d == p.head_dim and g == group
    dQ, dK, dV = to_dev(Q, sess.dtype), to_dev(K, sess.dtype), to_dev(V, sess.dtype)
    dlen = torch.tensor(list(lens), dtype=torch.int32, device="cuda")
    sess.prefill_ws = torch.empty(max(16, roco.prefill_gqa_workspace_bytes(p, group, L_max)), dtype=torch.uint8,
                                  device="cuda")
    c = sess.cache
    sess.O = torch.zeros_like(dQ) if want_out else None
    roco.roco_prefill_compress_gqa(p, group, dQ, dK, dV, dlen, L_max, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot,
                                   sess.O, sess.prefill_ws)
    torch.cuda.synchronize()
    return dict(K=to_host(c.K), V=to_host(c.V), stats=to_host(c.stats), pos=to_host(c.pos), n_used=to_host(c.n_used),
                O=None if sess.O is None else to_host(sess.O))
