"""Plain float64 NumPy oracle for RoCo (arxiv 2402.06262).  TEST INFRASTRUCTURE ONLY.

This file is the slow, obviously-correct statement of what the HIP library must
compute.  It is used by the tests, the smoke check and the CPU-baseline leg of
the benchmark, and by nothing in the product path.  It shares no code with the
HIP path and imports nothing from it.

RoCo is a heuristic applied step by step, not a shortcut to a closed-form
result, so the oracle is the algorithm itself, in the paper's order and
notation, on one *unit* (one attention head of one sequence of one layer; the
paper's Fig. 1 caption: every head evicts at its own positions):

* scaled dot-product attention per head, causal                 (section 2.1, eq. 1)
* a fixed buffer of at most B tokens per head, evict when full  (section 3,
  "Key-Value Constrained Inference"; section 4, first paragraph)
* importance = mean attention score, MAS = Acc / Count          (section 4.3, "Results")
* eviction scope from the standard deviation
      Std(x) = sqrt(Acc2(x)/Count(x) - (Acc(x)/Count(x))^2)
  of the attention probabilities a token has received: the tokens with the
  largest Std are kept out of the scope, and the token with the lowest MAS
  inside the scope is removed                                    (section 4.3, Std paragraph)
* Acc, Acc2 (the paper's Acc^square) and Count are three B-sized arrays per
  head                                                           (same paragraph; section 5.3 "Overhead")
* prefill eviction frees many tokens in one eviction step        (section 5.3 "Overhead", block-wise
  evict-and-encode; appendix B)

Readings taken where the paper is silent:

* `scope` = s = the number of tokens *inside* the eviction scope, i.e. the s
  occupied slots of smallest variance; the paper's r (number of protected
  top-Std tokens) is n - s.
* Ranking uses the population variance max(0, Acc2/Count - MAS^2); the square
  root is monotone and is not taken.
* One eviction step that frees E > 1 tokens is E token-wise RoCo evictions
  with the statistics frozen.  `select_evictions_literal` is that loop;
  `select_evictions` is its closed form (the E lowest-MAS tokens among the
  s + E - 1 lowest-variance tokens); the tests check they agree.
* A token's own query counts among the queries that attended it, so the key at
  position j of an L-token prompt has Count = L - j.
* Evict first, then append: the victim is chosen from the statistics of the
  previous steps, the new key/value overwrite its slot, and attention runs over
  at most B entries.
* Ties (equal variance at the scope boundary, equal MAS) go to the lowest slot
  index; before compaction slot index equals position.
* After prefill compaction the retained tokens are stored in ascending position.
* An optional recency bias adds `recency_bias` to the scaled logit when
  0 <= qpos - kpos < recency_window (workload 5 only; not from the paper).

PARITY PINS (tests/test_oracle_*.py): softmax rows sum to one; the cache never
exceeds B; B >= length reproduces dense causal attention written
independently; incremental statistics equal a brute-force recount from the
logged attention rows; two closed forms (uniform attention -> harmonic numbers;
one-dimensional log-weights -> exact rationals) including a hand-worked 6-token
example; closed-form selection equals the literal loop; slot-permutation
invariance of a decode step.
PARITY UNPINNED by the paper itself: the readings listed above (the paper prints
no numeric example of RoCo); they are pinned only by internal consistency.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

F64 = np.float64


# ---------------------------------------------------------------------------
# attention (section 2.1, eq. 1) with the causal mask (section 2.1, "Key-Value Cache")
# ---------------------------------------------------------------------------

def _recency(qpos: np.ndarray, kpos: np.ndarray, window: int, bias: float) -> np.ndarray:
    """bias * 1[0 <= qpos - kpos < window], broadcast qpos[:,None] against kpos[None,:]."""
    if window <= 0 or bias == 0.0:
        return np.zeros((qpos.shape[0], kpos.shape[0]), dtype=F64)
    diff = qpos[:, None] - kpos[None, :]
    return np.where((diff >= 0) & (diff < window), F64(bias), F64(0.0))


def causal_probability_rows(Q, K, length: int, scale: float, recency_window: int = 0,
                            recency_bias: float = 0.0, row_block: int = 512):
    """Yield (i0, P) with P[i - i0, j] = softmax_j(scale q_i.k_j + bias), j <= i < length.

    Entries with j > i are exactly zero.  Evaluated a block of query rows at a
    time only to bound memory; the values are those of the definition.
    """
    Q = np.asarray(Q, dtype=F64)[:length]
    K = np.asarray(K, dtype=F64)[:length]
    kpos = np.arange(length)
    for i0 in range(0, length, row_block):
        i1 = min(length, i0 + row_block)
        qpos = np.arange(i0, i1)
        S = (Q[i0:i1] @ K[:i1].T) * F64(scale)
        S = S + _recency(qpos, kpos[:i1], recency_window, recency_bias)
        visible = kpos[None, :i1] <= qpos[:, None]
        S = np.where(visible, S, -np.inf)
        S = S - S.max(axis=1, keepdims=True)
        P = np.exp(S)
        P = P / P.sum(axis=1, keepdims=True)
        yield i0, P


def row_log_sum_exp(Q, K, length: int, scale: float, recency_window: int = 0, recency_bias: float = 0.0,
                    row_block: int = 512) -> np.ndarray:
    """lse[i] = ln sum_{j <= i} exp(scale q_i.k_j + bias(i, j)), i < length: the normaliser of row i of the causal
    softmax (section 2.1, eq. 1), as an attention kernel hands it to a caller that wants the probabilities back
    (P[i, j] = exp(logit - lse[i])).  Natural logarithm.  Row blocks only bound memory."""
    Q = np.asarray(Q, dtype=F64)[:length]
    K = np.asarray(K, dtype=F64)[:length]
    kpos = np.arange(length)
    lse = np.empty(length, dtype=F64)
    for i0 in range(0, length, row_block):
        i1 = min(length, i0 + row_block)
        qpos = np.arange(i0, i1)
        S = (Q[i0:i1] @ K[:i1].T) * F64(scale) + _recency(qpos, kpos[:i1], recency_window, recency_bias)
        S = np.where(kpos[None, :i1] <= qpos[:, None], S, -np.inf)
        top = S.max(axis=1)
        lse[i0:i1] = top + np.log(np.exp(S - top[:, None]).sum(axis=1))
    return lse


@dataclass
class PrefillStats:
    acc: np.ndarray  # [length]  sum over queries i >= j of P[i, j]
    acc2: np.ndarray  # [length] sum over queries i >= j of P[i, j]^2
    count: np.ndarray  # [length] number of queries that attended key j = length - j
    out: Optional[np.ndarray]  # [length, d] attention output, if requested


def _keeps_last_score(policy) -> bool:
    """Whether the policy's second statistic is the last query's attention (importance "ltas") instead of the
    accumulated squared attention."""
    return policy is not None and policy.importance == "ltas"


def _counts_above_average(policy) -> bool:
    """Whether the policy's second statistic counts the queries whose attention to the token was above the
    row average (importance "aqas")."""
    return policy is not None and policy.importance == "aqas"


def above_average(p, n_attended):
    """The quantised attention score of section 4.1 (AQAS): 1 where a probability exceeds the average of its
    softmax row, i.e. 1 / (number of tokens the query attended), else 0."""
    return (np.asarray(p, dtype=F64) * F64(n_attended) > F64(1.0)).astype(F64)


def _second_statistic(policy, old, p, seen, n_attended):
    """The second array after a query with probabilities `p` over the slots flagged `seen` (p is 0 elsewhere)."""
    if _keeps_last_score(policy):
        return np.where(seen, p, old)
    if _counts_above_average(policy):
        return old + np.where(seen, above_average(p, n_attended), 0.0)
    return old + p * p


def prefill_statistics(Q, K, V, length: int, scale: float, recency_window: int = 0,
                       recency_bias: float = 0.0, want_out: bool = False,
                       row_block: int = 512, policy=None) -> PrefillStats:
    """Column statistics of the causal attention matrix (section 4.3: Acc, Acc^square, Count).

    Under the last-token importance score (section 4.1, LTAS) the second array holds the attention row of the
    last prompt token instead of the accumulated squares."""
    acc = np.zeros(length, dtype=F64)
    acc2 = np.zeros(length, dtype=F64)
    count = np.zeros(length, dtype=F64)
    Vd = np.asarray(V, dtype=F64)[:length]
    out = np.zeros((length, Vd.shape[1]), dtype=F64) if want_out else None
    for i0, P in causal_probability_rows(Q, K, length, scale, recency_window,
                                         recency_bias, row_block):
        i1 = i0 + P.shape[0]
        acc[:i1] += P.sum(axis=0)
        if _keeps_last_score(policy):
            if i0 <= length - 1 < i1:
                acc2[:i1] = P[length - 1 - i0]
        elif _counts_above_average(policy):
            causal = np.arange(i1)[None, :] <= np.arange(i0, i1)[:, None]
            acc2[:i1] += (causal & (P * np.arange(i0 + 1, i1 + 1, dtype=F64)[:, None] > 1.0)).sum(axis=0)
        else:
            acc2[:i1] += (P * P).sum(axis=0)
        count[:i1] += (np.arange(i1)[None, :] <= np.arange(i0, i1)[:, None]).sum(axis=0)
        if want_out:
            out[i0:i1] = P @ Vd[:i1]
    return PrefillStats(acc, acc2, count, out)


# ---------------------------------------------------------------------------
# importance and robustness measures (section 4.3)
# ---------------------------------------------------------------------------

def mean_attention_score(acc, count):
    """MAS = Acc / Count."""
    return np.asarray(acc, dtype=F64) / np.asarray(count, dtype=F64)


def attention_variance(acc, acc2, count):
    """Std(x)^2 = Acc2/Count - (Acc/Count)^2, clamped at zero."""
    acc, acc2, count = (np.asarray(a, dtype=F64) for a in (acc, acc2, count))
    mas = acc / count
    return np.maximum(F64(0.0), acc2 / count - mas * mas)


def k_smallest(values: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k smallest values; equal values are taken in index order."""
    order = np.argsort(np.asarray(values, dtype=F64), kind="stable")
    return np.sort(order[:k])


def select_victim(mas: np.ndarray, var: np.ndarray, scope: int) -> int:
    """One RoCo eviction: scope = the `scope` lowest-variance tokens, victim = lowest MAS in it."""
    inside = k_smallest(var, scope)
    return int(inside[np.argmin(mas[inside])])  # argmin returns the first (lowest index) minimum


def select_evictions_literal(mas: np.ndarray, var: np.ndarray, scope: int, n_evict: int) -> np.ndarray:
    """E token-wise evictions with frozen statistics, one at a time (the literal reading)."""
    alive = np.ones(mas.shape[0], dtype=bool)
    victims: List[int] = []
    for _ in range(n_evict):
        idx = np.flatnonzero(alive)
        v = idx[select_victim(mas[idx], var[idx], min(scope, idx.shape[0]))]
        victims.append(int(v))
        alive[v] = False
    return np.sort(np.array(victims, dtype=np.int64))


def select_evictions(mas: np.ndarray, var: np.ndarray, scope: int, n_evict: int) -> np.ndarray:
    """Closed form of the loop above: the E lowest-MAS among the s+E-1 lowest-variance tokens."""
    if n_evict <= 0:
        return np.zeros(0, dtype=np.int64)
    eligible = k_smallest(var, min(mas.shape[0], scope + n_evict - 1))
    return np.sort(eligible[k_smallest(mas[eligible], n_evict)])


# ---------------------------------------------------------------------------
# other eviction policies in the same two-stage framework (section 4: an eviction scope, then an importance
# score inside it; section 4.1 lists the importance scores, section 4.2 / 4.3 the scopes)
# ---------------------------------------------------------------------------

@dataclass(frozen=True)
class Policy:
    """importance: "mas" (Acc/Count, section 4.3), "aas" (accumulated attention score Acc, the H2O score of
    section 4.1), "oldest" (recency: the lowest position goes first, except the first `sinks` positions, which
    are never chosen while anything else is in scope: the window / StreamLLM baseline of section 4.1), "ltas"
    (the attention the token received from the most recent query, the TOVA score of section 4.1; the array that
    otherwise accumulates squared attention then holds that score, so the "std" scope is not available), "aqas"
    (the number of queries that gave the token more than the average attention of their row, the quantised score
    of section 4.1 (ScissorHands); it too lives in the second array).
    scope_kind: "std" (the s tokens of lowest variance, section 4.3), "window" (the s oldest tokens, i.e. the
    most recent n - s are protected: the local-window scope of section 4.2), "all" (every cached token)."""
    importance: str = "mas"
    scope_kind: str = "std"
    sinks: int = 0


ROCO = Policy()


def ranking_scores(policy: Optional[Policy], acc, acc2, count, pos, scope: int):
    """(importance, scope key, scope size) of every cached token under `policy`; None is RoCo.

    Lower importance is evicted first; the scope is the `scope size` tokens of lowest scope key (ties by index).
    """
    policy = policy or ROCO
    acc, acc2, count = (np.asarray(a, dtype=F64) for a in (acc, acc2, count))
    pos = np.asarray(pos)
    n = acc.shape[0]
    if policy.importance == "mas":
        importance = mean_attention_score(acc, count)
    elif policy.importance == "aas":
        importance = acc.copy()
    elif policy.importance == "oldest":
        importance = np.where(pos < policy.sinks, np.inf, pos.astype(F64))
    elif policy.importance in ("ltas", "aqas"):
        if policy.scope_kind == "std":
            raise ValueError("the last-token score replaces the squared-attention array: no variance to rank by")
        importance = acc2.copy()
    else:
        raise ValueError(policy.importance)
    if policy.scope_kind == "std":
        return importance, attention_variance(acc, acc2, count), scope
    if policy.scope_kind == "window":
        return importance, pos.astype(F64), scope
    if policy.scope_kind == "all":
        return importance, np.zeros(n, dtype=F64), n
    raise ValueError(policy.scope_kind)


# ---------------------------------------------------------------------------
# the two calls of the boundary
# ---------------------------------------------------------------------------

@dataclass
class CacheState:
    """Budgeted per-head cache: at most `budget` slots (section 3: n <= B at every step)."""

    K: np.ndarray  # [budget, d] float64
    V: np.ndarray  # [budget, d]
    acc: np.ndarray  # [budget]
    acc2: np.ndarray  # [budget]
    count: np.ndarray  # [budget]
    pos: np.ndarray  # [budget] int64 original position, -1 for an empty slot
    n_used: int

    @property
    def budget(self) -> int:
        return self.K.shape[0]

    def copy(self) -> "CacheState":
        return CacheState(self.K.copy(), self.V.copy(), self.acc.copy(), self.acc2.copy(),
                          self.count.copy(), self.pos.copy(), self.n_used)


@dataclass
class PrefillResult:
    cache: CacheState
    out: Optional[np.ndarray]  # [length, d] or None
    full: PrefillStats  # statistics of all prompt tokens before eviction
    evicted: np.ndarray  # sorted positions removed
    retained: np.ndarray  # sorted positions kept


def compress_from_statistics(full: PrefillStats, K, V, length: int, budget: int, scope: int,
                             force_retained: Optional[np.ndarray] = None,
                             policy: Optional[Policy] = None) -> PrefillResult:
    """The eviction step and the compaction of `prefill_compress`, given the prompt's statistics."""
    n_evict = max(0, length - budget)
    mas, var, s_eff = ranking_scores(policy, full.acc, full.acc2, full.count, np.arange(length), scope)
    evicted = select_evictions(mas, var, s_eff, n_evict)
    keep = np.ones(length, dtype=bool)
    keep[evicted] = False
    retained = np.flatnonzero(keep)
    if force_retained is not None:
        retained = np.sort(np.asarray(force_retained, dtype=np.int64))
        keep[:] = False
        keep[retained] = True
        evicted = np.flatnonzero(~keep)
    n = retained.shape[0]
    assert n == min(length, budget)
    d = np.asarray(K).shape[1]
    cache = CacheState(np.zeros((budget, d), F64), np.zeros((budget, d), F64),
                       np.zeros(budget, F64), np.zeros(budget, F64), np.zeros(budget, F64),
                       np.full(budget, -1, dtype=np.int64), n)
    cache.K[:n] = np.asarray(K, dtype=F64)[retained]
    cache.V[:n] = np.asarray(V, dtype=F64)[retained]
    cache.acc[:n] = full.acc[retained]
    cache.acc2[:n] = full.acc2[retained]
    cache.count[:n] = full.count[retained]
    cache.pos[:n] = retained
    return PrefillResult(cache, full.out, full, evicted, retained)


def prefill_compress(Q, K, V, length: int, budget: int, scope: int, scale: float,
                     recency_window: int = 0, recency_bias: float = 0.0,
                     want_out: bool = False, row_block: int = 512,
                     force_retained: Optional[np.ndarray] = None,
                     policy: Optional[Policy] = None) -> PrefillResult:
    """Encode a prompt and compress its cache to `budget` tokens in one eviction step.

    `force_retained` replaces the oracle's own retained set (used by the parity
    harness after a declared tie, never by the pins).
    """
    full = prefill_statistics(Q, K, V, length, scale, recency_window, recency_bias,
                              want_out, row_block, policy)
    return compress_from_statistics(full, K, V, length, budget, scope, force_retained, policy)


@dataclass
class DecodeResult:
    out: np.ndarray  # [d]
    probs: np.ndarray  # [n_used] attention probabilities over the occupied slots
    evicted_slot: int  # -1 when nothing was evicted
    evicted_pos: int
    written_slot: int
    mas: Optional[np.ndarray]  # statistics the decision was taken on (None if no eviction)
    var: Optional[np.ndarray]


def decode_step(state: CacheState, q, k_new, v_new, qpos: int, scope: int, scale: float,
                recency_window: int = 0, recency_bias: float = 0.0,
                force_victim: Optional[int] = None, policy: Optional[Policy] = None) -> DecodeResult:
    """One auto-regressive step on a budgeted cache, in place: evict, append, attend, update."""
    B = state.budget
    mas = var = None
    if state.n_used == B:
        mas, var, s_eff = ranking_scores(policy, state.acc, state.acc2, state.count, state.pos, scope)
        slot = select_victim(mas, var, s_eff) if force_victim is None else int(force_victim)
        evicted_slot, evicted_pos = slot, int(state.pos[slot])
    else:
        slot = state.n_used
        state.n_used += 1
        evicted_slot, evicted_pos = -1, -1
    state.K[slot] = np.asarray(k_new, dtype=F64)
    state.V[slot] = np.asarray(v_new, dtype=F64)
    state.pos[slot] = qpos
    state.acc[slot] = state.acc2[slot] = state.count[slot] = 0.0
    n = state.n_used
    z = (state.K[:n] @ np.asarray(q, dtype=F64)) * F64(scale)
    z = z + _recency(np.array([qpos]), state.pos[:n], recency_window, recency_bias)[0]
    p = np.exp(z - z.max())
    p = p / p.sum()
    out = p @ state.V[:n]
    state.acc[:n] += p
    state.acc2[:n] = _second_statistic(policy, state.acc2[:n], p, np.ones(n, dtype=bool), n)
    state.count[:n] += 1.0
    return DecodeResult(out, p, evicted_slot, evicted_pos, slot, mas, var)


# ---------------------------------------------------------------------------
# block-wise evict-and-encode (section 5.3 "Overhead"; appendix B)
# ---------------------------------------------------------------------------

@dataclass
class BlockResult:
    out: np.ndarray  # [b, d]
    probs: List[np.ndarray]  # probs[i][slot]: attention of the block's i-th query over the slots (0 where unseen)
    slots: np.ndarray  # [b] slot each block token was written to
    evicted_slot: np.ndarray  # [b] = slots[i] if that slot held a token that was evicted, else -1
    evicted_pos: np.ndarray  # [b] position of that evicted token, else -1
    mas: Optional[np.ndarray]  # statistics the decision was taken on (None if nothing was evicted)
    var: Optional[np.ndarray]


def encode_block(state: CacheState, Qb, Kb, Vb, qpos0: int, scope: int, scale: float,
                 recency_window: int = 0, recency_bias: float = 0.0,
                 force_evicted: Optional[np.ndarray] = None, policy: Optional[Policy] = None) -> BlockResult:
    """Free and encode b tokens within one eviction step, in place.

    The paper lets the number of tokens freed and encoded per eviction step be a block size b (section 5.3;
    b = 1 is the token-wise scheme).  Reading taken here: with n tokens in the cache, E = max(0, n + b - B)
    tokens are evicted in one step from the statistics as they stand (E single evictions with frozen
    statistics, i.e. `select_evictions`); the block's tokens go, in order, to the ascending list of freed and
    still-empty slots; query i of the block attends every retained token and the block's tokens 0..i; every
    attended token gets p, p^2 and 1 added to its three statistics.  b = 1 is exactly `decode_step`.
    """
    Qb, Kb, Vb = (np.asarray(x, dtype=F64) for x in (Qb, Kb, Vb))
    b = Qb.shape[0]
    B, n = state.budget, state.n_used
    assert 1 <= b <= B
    E = max(0, n + b - B)
    mas = var = None
    evicted = np.zeros(0, dtype=np.int64)
    if E > 0:
        mas, var, s_eff = ranking_scores(policy, state.acc[:n], state.acc2[:n], state.count[:n], state.pos[:n], scope)
        evicted = select_evictions(mas, var, s_eff, E) if force_evicted is None else \
            np.sort(np.asarray(force_evicted, dtype=np.int64))
    targets = np.sort(np.concatenate([evicted, np.arange(n, min(B, n + b), dtype=np.int64)]))
    assert targets.shape[0] == b
    was_evicted = np.isin(targets, evicted)
    evicted_slot = np.where(was_evicted, targets, -1)
    evicted_pos = np.where(was_evicted, state.pos[targets], -1)
    block_index = np.full(B, -1, dtype=np.int64)  # which block token sits in a slot, -1 for older tokens
    for i, slot in enumerate(targets):
        state.K[slot], state.V[slot] = Kb[i], Vb[i]
        state.pos[slot] = qpos0 + i
        state.acc[slot] = state.acc2[slot] = state.count[slot] = 0.0
        block_index[slot] = i
    state.n_used = n_new = min(B, n + b)
    out = np.zeros((b, Vb.shape[1]), dtype=F64)
    probs = []
    for i in range(b):
        seen = np.flatnonzero(block_index[:n_new] <= i)  # older tokens (-1) and block tokens 0..i
        z = (state.K[seen] @ Qb[i]) * F64(scale)
        z = z + _recency(np.array([qpos0 + i]), state.pos[seen], recency_window, recency_bias)[0]
        p = np.exp(z - z.max())
        p = p / p.sum()
        out[i] = p @ state.V[seen]
        full = np.zeros(n_new, dtype=F64)
        full[seen] = p
        probs.append(full)
    for i in range(b):  # statistics after all rows are known, in the block's order
        state.acc[:n_new] += probs[i]
        seen = block_index[:n_new] <= i
        state.acc2[:n_new] = _second_statistic(policy, state.acc2[:n_new], probs[i], seen, int(seen.sum()))
        state.count[:n_new] += seen.astype(F64)
    return BlockResult(out, probs, targets, evicted_slot, evicted_pos, mas, var)


# ---------------------------------------------------------------------------
# grouped-query attention (section 5.3 "Extension to Grouped-Query Attention"; appendix A)
# ---------------------------------------------------------------------------

@dataclass
class GroupDecodeResult:
    out: np.ndarray  # [g, d] one attention output per query head of the group
    probs: np.ndarray  # [g, n_used]
    mean_probs: np.ndarray  # [n_used] group-wise averaged attention: what the statistics receive
    evicted_slot: int
    evicted_pos: int
    written_slot: int
    mas: Optional[np.ndarray]
    var: Optional[np.ndarray]


def decode_step_gqa(state: CacheState, Qg, k_new, v_new, qpos: int, scope: int, scale: float,
                    recency_window: int = 0, recency_bias: float = 0.0,
                    force_victim: Optional[int] = None, policy: Optional[Policy] = None) -> GroupDecodeResult:
    """One decode step of a key/value head shared by g query heads.

    The paper extends attention-based policies to GQA / MQA by updating the importance score with the group-wise
    averaged attention score.  Here: every query head of the group attends the shared cache as usual; the cache's
    statistics receive the mean of the g probability vectors (Acc += mean p, Acc2 += (mean p)^2, Count += 1).
    The eviction rule is unchanged.  g = 1 is exactly `decode_step`.
    """
    Qg = np.asarray(Qg, dtype=F64)
    g = Qg.shape[0]
    B = state.budget
    mas = var = None
    if state.n_used == B:
        mas, var, s_eff = ranking_scores(policy, state.acc, state.acc2, state.count, state.pos, scope)
        slot = select_victim(mas, var, s_eff) if force_victim is None else int(force_victim)
        evicted_slot, evicted_pos = slot, int(state.pos[slot])
    else:
        slot = state.n_used
        state.n_used += 1
        evicted_slot, evicted_pos = -1, -1
    state.K[slot] = np.asarray(k_new, dtype=F64)
    state.V[slot] = np.asarray(v_new, dtype=F64)
    state.pos[slot] = qpos
    state.acc[slot] = state.acc2[slot] = state.count[slot] = 0.0
    n = state.n_used
    bias = _recency(np.array([qpos]), state.pos[:n], recency_window, recency_bias)[0]
    probs = np.zeros((g, n), dtype=F64)
    out = np.zeros((g, state.V.shape[1]), dtype=F64)
    for h in range(g):
        z = (state.K[:n] @ Qg[h]) * F64(scale) + bias
        p = np.exp(z - z.max())
        probs[h] = p / p.sum()
        out[h] = probs[h] @ state.V[:n]
    mean_p = probs.sum(axis=0) / F64(g)
    state.acc[:n] += mean_p
    state.acc2[:n] = _second_statistic(policy, state.acc2[:n], mean_p, np.ones(n, dtype=bool), n)
    state.count[:n] += 1.0
    return GroupDecodeResult(out, probs, mean_p, evicted_slot, evicted_pos, slot, mas, var)


@dataclass
class GroupBlockResult:
    out: np.ndarray  # [b, g, d]
    mean_probs: List[np.ndarray]  # mean_probs[i][slot]: group-wise averaged attention of block token i (0 where unseen)
    slots: np.ndarray
    evicted_slot: np.ndarray
    evicted_pos: np.ndarray
    mas: Optional[np.ndarray]
    var: Optional[np.ndarray]


def encode_block_gqa(state: CacheState, Qb, Kb, Vb, qpos0: int, scope: int, scale: float,
                     recency_window: int = 0, recency_bias: float = 0.0,
                     force_evicted: Optional[np.ndarray] = None, policy: Optional[Policy] = None) -> GroupBlockResult:
    """Block-wise evict-and-encode of a key/value head shared by g query heads: Qb is [b, g, d], Kb / Vb [b, d].

    Eviction and slot assignment exactly as in `encode_block`; token i of the block is attended from by its g
    query heads, each over the retained tokens and the block's tokens 0..i, and the statistics receive the mean of
    those g probability vectors once per token (section 5.3, both extensions together).  g = 1 is `encode_block`,
    b = 1 is `decode_step_gqa`.
    """
    Qb, Kb, Vb = (np.asarray(x, dtype=F64) for x in (Qb, Kb, Vb))
    b, g = Qb.shape[0], Qb.shape[1]
    B, n = state.budget, state.n_used
    assert 1 <= b <= B
    E = max(0, n + b - B)
    mas = var = None
    evicted = np.zeros(0, dtype=np.int64)
    if E > 0:
        mas, var, s_eff = ranking_scores(policy, state.acc[:n], state.acc2[:n], state.count[:n], state.pos[:n], scope)
        evicted = select_evictions(mas, var, s_eff, E) if force_evicted is None else \
            np.sort(np.asarray(force_evicted, dtype=np.int64))
    targets = np.sort(np.concatenate([evicted, np.arange(n, min(B, n + b), dtype=np.int64)]))
    assert targets.shape[0] == b
    was_evicted = np.isin(targets, evicted)
    evicted_slot = np.where(was_evicted, targets, -1)
    evicted_pos = np.where(was_evicted, state.pos[targets], -1)
    block_index = np.full(B, -1, dtype=np.int64)
    for i, slot in enumerate(targets):
        state.K[slot], state.V[slot] = Kb[i], Vb[i]
        state.pos[slot] = qpos0 + i
        state.acc[slot] = state.acc2[slot] = state.count[slot] = 0.0
        block_index[slot] = i
    state.n_used = n_new = min(B, n + b)
    out = np.zeros((b, g, Vb.shape[1]), dtype=F64)
    means = []
    for i in range(b):
        seen = np.flatnonzero(block_index[:n_new] <= i)
        bias = _recency(np.array([qpos0 + i]), state.pos[seen], recency_window, recency_bias)[0]
        total = np.zeros(seen.shape[0], dtype=F64)
        for h in range(g):
            z = (state.K[seen] @ Qb[i, h]) * F64(scale) + bias
            p = np.exp(z - z.max())
            p = p / p.sum()
            out[i, h] = p @ state.V[seen]
            total += p
        full = np.zeros(n_new, dtype=F64)
        full[seen] = total / F64(g)
        means.append(full)
    for i in range(b):
        state.acc[:n_new] += means[i]
        seen = block_index[:n_new] <= i
        state.acc2[:n_new] = _second_statistic(policy, state.acc2[:n_new], means[i], seen, int(seen.sum()))
        state.count[:n_new] += seen.astype(F64)
    return GroupBlockResult(out, means, targets, evicted_slot, evicted_pos, mas, var)


# ---------------------------------------------------------------------------
# which tokens a smaller budget would keep (the sets compared in section 4.1's consistency study)
# ---------------------------------------------------------------------------

def select_retained(state: CacheState, keep: int, scope: int, policy: Optional[Policy] = None) -> np.ndarray:
    """Boolean mask over the slots: the cached tokens that survive one eviction step shrinking the cache to
    `keep` tokens (n_used - keep evictions with the statistics as they stand; nothing is changed).

    With scope "all" these are the `keep` most important cached tokens: the "top-B important tokens" whose
    overlap between a budgeted and a full cache section 4.1 measures (Jaccard similarity)."""
    n = state.n_used
    mask = np.zeros(state.budget, dtype=bool)
    mask[:n] = True
    if n > keep:
        imp, key, s_eff = ranking_scores(policy, state.acc[:n], state.acc2[:n], state.count[:n], state.pos[:n], scope)
        mask[select_evictions(imp, key, s_eff, n - keep)] = False
    return mask


# ---------------------------------------------------------------------------
# grouped-query prefill: the prompt of a key/value head shared by g query heads
# ---------------------------------------------------------------------------

def prefill_statistics_gqa(Qg, K, V, length: int, scale: float, recency_window: int = 0,
                           recency_bias: float = 0.0, row_block: int = 512, policy=None,
                           want_out: bool = False) -> PrefillStats:
    """Column statistics of the group-wise averaged causal attention matrix: Qg is [g, length, d].

    Every query head has its own causal softmax (section 2.1, eq. 1); the statistics of the shared key/value
    head are taken on the mean of the g probability matrices (section 5.3, grouped-query extension):
    Acc[j] = sum_i Pbar[i,j], Acc2[j] = sum_i Pbar[i,j]^2 (or the last row of Pbar under the last-token score),
    Count[j] = length - j.  `out`, if asked for, is [g, length, d]: every head's own attention output."""
    Qg = np.asarray(Qg, dtype=F64)
    g = Qg.shape[0]
    acc = np.zeros(length, dtype=F64)
    acc2 = np.zeros(length, dtype=F64)
    count = np.zeros(length, dtype=F64)
    Vd = np.asarray(V, dtype=F64)[:length]
    out = np.zeros((g, length, Vd.shape[1]), dtype=F64) if want_out else None
    rows = [causal_probability_rows(Qg[h], K, length, scale, recency_window, recency_bias, row_block) for h in range(g)]
    for blocks in zip(*rows):
        i0 = blocks[0][0]
        Pbar = sum(P for _, P in blocks) / F64(g)
        i1 = i0 + Pbar.shape[0]
        if want_out:
            for h, (_, P) in enumerate(blocks):
                out[h, i0:i1] = P @ Vd[:i1]
        acc[:i1] += Pbar.sum(axis=0)
        if _keeps_last_score(policy):
            if i0 <= length - 1 < i1:
                acc2[:i1] = Pbar[length - 1 - i0]
        elif _counts_above_average(policy):
            causal = np.arange(i1)[None, :] <= np.arange(i0, i1)[:, None]
            acc2[:i1] += (causal & (Pbar * np.arange(i0 + 1, i1 + 1, dtype=F64)[:, None] > 1.0)).sum(axis=0)
        else:
            acc2[:i1] += (Pbar * Pbar).sum(axis=0)
        count[:i1] += (np.arange(i1)[None, :] <= np.arange(i0, i1)[:, None]).sum(axis=0)
    return PrefillStats(acc, acc2, count, out)


def prefill_compress_gqa(Qg, K, V, length: int, budget: int, scope: int, scale: float,
                         recency_window: int = 0, recency_bias: float = 0.0, row_block: int = 512,
                         force_retained: Optional[np.ndarray] = None, policy: Optional[Policy] = None) -> PrefillResult:
    """`prefill_compress` for a key/value head shared by g query heads (Qg is [g, length, d])."""
    full = prefill_statistics_gqa(Qg, K, V, length, scale, recency_window, recency_bias, row_block, policy)
    return compress_from_statistics(full, K, V, length, budget, scope, force_retained, policy)
