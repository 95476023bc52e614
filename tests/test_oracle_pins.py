"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle's code.

Every expected value here comes from a closed form, an exact rational computation, a brute-force
recount, or a textbook routine written separately -- never from the oracle itself.
"""
import itertools
import math
import os
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import roco_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "six_token_example.txt")


def load_golden():
    rec = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rec[key] = [Fr(v) for v in vals]
    return rec


def dense_causal_attention(Q, K, V, scale):
    """Textbook dense causal attention (section 2.1 eq. 1), written independently of the oracle."""
    L = Q.shape[0]
    S = np.einsum("id,jd->ij", Q, K) * scale
    S[np.triu_indices(L, 1)] = -np.inf
    E = np.exp(S - S.max(1)[:, None])
    P = E / E.sum(1)[:, None]
    return P, P @ V


def rand_unit(rng, T, d):
    return rng.standard_normal((T, d)), rng.standard_normal((T, d)), rng.standard_normal((T, d))


# ---------------------------------------------------------------------------- invariants

def test_rows_sum_to_one_and_are_causal():
    rng = np.random.default_rng(1)
    Q, K, _ = rand_unit(rng, 70, 8)
    seen = 0
    for i0, P in orc.causal_probability_rows(Q, K, 70, 0.35, row_block=16):
        assert np.allclose(P.sum(1), 1.0, atol=1e-12)
        for r in range(P.shape[0]):
            assert np.all(P[r, i0 + r + 1:] == 0.0)
            assert np.all(P[r, : i0 + r + 1] > 0.0)
        seen += P.shape[0]
    assert seen == 70


def test_row_block_size_does_not_change_values():
    rng = np.random.default_rng(2)
    Q, K, V = rand_unit(rng, 45, 4)
    a = orc.prefill_statistics(Q, K, V, 45, 0.5, want_out=True, row_block=7)
    b = orc.prefill_statistics(Q, K, V, 45, 0.5, want_out=True, row_block=512)
    for x, y in ((a.acc, b.acc), (a.acc2, b.acc2), (a.count, b.count), (a.out, b.out)):
        assert np.allclose(x, y, rtol=1e-13, atol=1e-15)


def test_prefill_matches_independent_dense_attention():
    rng = np.random.default_rng(3)
    L, d = 37, 6
    Q, K, V = rand_unit(rng, L, d)
    P, O = dense_causal_attention(Q, K, V, 1 / math.sqrt(d))
    st = orc.prefill_statistics(Q, K, V, L, 1 / math.sqrt(d), want_out=True)
    assert np.allclose(st.out, O, rtol=1e-12, atol=1e-14)
    assert np.allclose(st.acc, P.sum(0), rtol=1e-12)
    assert np.allclose(st.acc2, (P ** 2).sum(0), rtol=1e-12)
    assert np.array_equal(st.count, L - np.arange(L))  # a token's own query counts


def test_length_shorter_than_arrays_ignores_the_tail():
    rng = np.random.default_rng(4)
    Q, K, V = rand_unit(rng, 30, 4)
    a = orc.prefill_statistics(Q, K, V, 19, 0.5, want_out=True)
    b = orc.prefill_statistics(Q[:19], K[:19], V[:19], 19, 0.5, want_out=True)
    assert np.array_equal(a.acc, b.acc) and np.array_equal(a.out, b.out)


def test_budget_at_least_length_reproduces_full_attention_and_never_evicts():
    rng = np.random.default_rng(5)
    L, steps, d = 20, 9, 5
    T = L + steps
    Q, K, V = rand_unit(rng, T, d)
    scale = 1 / math.sqrt(d)
    P, O = dense_causal_attention(Q, K, V, scale)
    res = orc.prefill_compress(Q[:L], K[:L], V[:L], L, T, 3, scale, want_out=True)
    assert res.evicted.size == 0 and res.cache.n_used == L
    assert np.allclose(res.out, O[:L], rtol=1e-12, atol=1e-14)
    for t in range(L, T):
        r = orc.decode_step(res.cache, Q[t], K[t], V[t], t, 3, scale)
        assert r.evicted_slot == -1 and r.evicted_pos == -1
        assert np.allclose(r.out, O[t], rtol=1e-12, atol=1e-14)
        assert res.cache.n_used == t + 1
    n = res.cache.n_used
    assert np.array_equal(res.cache.pos[:n], np.arange(T))
    assert np.allclose(res.cache.acc[:n], P.sum(0), rtol=1e-12)
    assert np.allclose(res.cache.acc2[:n], (P ** 2).sum(0), rtol=1e-12)
    assert np.array_equal(res.cache.count[:n], T - np.arange(T))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cache_never_exceeds_budget_and_incremental_stats_equal_brute_force(seed):
    """Log every attention row with the positions it covered; recount Acc, Acc2, Count per survivor."""
    rng = np.random.default_rng(100 + seed)
    L, steps, d, B, s = 24, 30, 4, 10, 3
    Q, K, V = rand_unit(rng, L + steps, d)
    scale = 0.7
    log = []  # (query position, {key position: probability})
    for i0, P in orc.causal_probability_rows(Q, K, L, scale, row_block=5):
        for r in range(P.shape[0]):
            i = i0 + r
            log.append((i, {j: P[r, j] for j in range(i + 1)}))
    res = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, scale)
    cache = res.cache
    assert cache.n_used == B and len(res.evicted) == L - B
    assert len(set(res.evicted) | set(res.retained)) == L
    for t in range(L, L + steps):
        before = cache.pos.copy()
        r = orc.decode_step(cache, Q[t], K[t], V[t], t, s, scale)
        assert cache.n_used <= B
        assert r.evicted_slot >= 0 and r.evicted_pos == before[r.evicted_slot]
        assert cache.pos[r.evicted_slot] == t
        assert abs(r.probs.sum() - 1.0) < 1e-12
        log.append((t, {int(cache.pos[j]): r.probs[j] for j in range(cache.n_used)}))
        # attention output equals softmax over exactly the cached keys, written independently
        z = np.array([scale * np.dot(Q[t], K[int(p)]) for p in cache.pos[:cache.n_used]])
        w = np.exp(z - z.max())
        w /= w.sum()
        assert np.allclose(r.out, sum(w[j] * V[int(cache.pos[j])] for j in range(cache.n_used)),
                           rtol=1e-12, atol=1e-14)
    assert len(set(cache.pos.tolist())) == B
    for j in range(B):
        p = int(cache.pos[j])
        rows = [row[p] for (i, row) in log if i >= p and p in row]
        assert cache.count[j] == len(rows)
        assert math.isclose(cache.acc[j], math.fsum(rows), rel_tol=1e-12)
        assert math.isclose(cache.acc2[j], math.fsum(x * x for x in rows), rel_tol=1e-12)
        assert np.array_equal(cache.K[j], K[p]) and np.array_equal(cache.V[j], V[p])


# ---------------------------------------------------------------------------- closed forms

@pytest.mark.parametrize("L", [1, 2, 17, 300])
def test_uniform_attention_gives_harmonic_numbers(L):
    """Q = 0 makes every causal row uniform: P[i,j] = 1/(i+1)."""
    rng = np.random.default_rng(L)
    K, V = rng.standard_normal((L, 3)), rng.standard_normal((L, 3))
    st = orc.prefill_statistics(np.zeros((L, 3)), K, V, L, 0.9, want_out=True)
    acc = [float(sum(Fr(1, i + 1) for i in range(j, L))) for j in range(L)]
    acc2 = [float(sum(Fr(1, (i + 1) ** 2) for i in range(j, L))) for j in range(L)]
    assert np.allclose(st.acc, acc, rtol=1e-12)
    assert np.allclose(st.acc2, acc2, rtol=1e-12)
    assert np.array_equal(st.count, [L - j for j in range(L)])
    running_mean = np.cumsum(V, 0) / np.arange(1, L + 1)[:, None]
    assert np.allclose(st.out, running_mean, rtol=1e-11, atol=1e-13)


def rational_case(w, scale):
    """d = 1, q_i = 1, k_j = ln(w_j)/scale  =>  P[i,j] = w_j / sum_{j'<=i} w_j' exactly."""
    L = len(w)
    Q = np.ones((L, 1))
    K = (np.log(np.array(w, dtype=np.float64)) / scale)[:, None]
    P = [[Fr(w[j], sum(w[: i + 1])) if j <= i else Fr(0) for j in range(L)] for i in range(L)]
    return Q, K, P


@pytest.mark.parametrize("scale", [1.0, 0.125, 3.0])
def test_log_weight_keys_give_exact_rationals(scale):
    w = [3, 1, 4, 1, 5, 9, 2, 6, 5, 3, 5]
    L = len(w)
    Q, K, P = rational_case(w, scale)
    V = np.arange(1, L + 1, dtype=np.float64)[:, None] * np.array([[1.0, -2.0]])
    st = orc.prefill_statistics(Q, K, V, L, scale, want_out=True)
    for j in range(L):
        assert math.isclose(st.acc[j], float(sum(P[i][j] for i in range(L))), rel_tol=1e-12)
        assert math.isclose(st.acc2[j], float(sum(P[i][j] ** 2 for i in range(L))), rel_tol=1e-12)
    for i in range(L):
        o = float(sum(P[i][j] * (j + 1) for j in range(L)))
        assert math.isclose(st.out[i, 0], o, rel_tol=1e-12)
        assert math.isclose(st.out[i, 1], -2 * o, rel_tol=1e-12)


def test_hand_worked_six_token_example():
    g = load_golden()
    w = [int(x) for x in g["w"]]
    L = len(w)
    Q, K, P = rational_case(w, 1.0)
    # the fixture is self-consistent with the closed form (checks the hand computation)
    for i in range(L):
        assert g[f"row{i}"] == P[i][: i + 1]
    assert g["acc"] == [sum(P[i][j] for i in range(L)) for j in range(L)]
    assert g["acc2"] == [sum(P[i][j] ** 2 for i in range(L)) for j in range(L)]
    assert g["mas"] == [a / c for a, c in zip(g["acc"], g["count"])]
    assert g["var"] == [a2 / c - m * m for a2, c, m in zip(g["acc2"], g["count"], g["mas"])]
    # the oracle reproduces it
    V = np.arange(1, L + 1, dtype=np.float64)[:, None]
    B, s = int(g["budget"][0]), int(g["scope"][0])
    res = orc.prefill_compress(Q, K, V, L, B, s, 1.0, want_out=True)
    f = lambda xs: np.array([float(x) for x in xs])  # noqa: E731
    assert np.allclose(res.full.acc, f(g["acc"]), rtol=1e-13)
    assert np.allclose(res.full.acc2, f(g["acc2"]), rtol=1e-13)
    assert np.array_equal(res.full.count, f(g["count"]))
    assert np.allclose(orc.mean_attention_score(res.full.acc, res.full.count), f(g["mas"]), rtol=1e-13)
    assert np.allclose(orc.attention_variance(res.full.acc, res.full.acc2, res.full.count),
                       f(g["var"]), rtol=1e-9, atol=1e-16)
    assert res.evicted.tolist() == [int(x) for x in g["evicted"]]
    assert res.retained.tolist() == [int(x) for x in g["retained"]]
    assert res.cache.pos.tolist() == [int(x) for x in g["retained"]]
    var = orc.attention_variance(res.full.acc, res.full.acc2, res.full.count)
    m = s + (L - B) - 1
    assert orc.k_smallest(var, m).tolist() == [int(x) for x in g["eligible"]]
    lit = orc.select_evictions_literal(orc.mean_attention_score(res.full.acc, res.full.count), var, s, L - B)
    assert lit.tolist() == [int(x) for x in g["evicted"]]
    # one decode step
    r = orc.decode_step(res.cache, [1.0], [math.log(float(g["decode_w"][0]))], [7.0], 6, s, 1.0)
    assert r.evicted_slot == int(g["decode_evicted_slot"][0])
    assert r.evicted_pos == int(g["decode_evicted_pos"][0])
    assert np.allclose(r.probs, f(g["decode_probs"]), rtol=1e-13)
    assert math.isclose(r.out[0], float(g["decode_out"][0]), rel_tol=1e-13)
    assert res.cache.pos.tolist() == [0, 6, 3]
    assert np.allclose(res.cache.acc, f(g["decode_acc"]), rtol=1e-13)
    assert np.allclose(res.cache.acc2, f(g["decode_acc2"]), rtol=1e-13)
    assert np.array_equal(res.cache.count, f(g["decode_count"]))


def test_recency_bias_with_a_huge_bias_becomes_window_attention():
    """bias = +80 on the last w positions (self included) leaves exp(-80) elsewhere."""
    rng = np.random.default_rng(7)
    L, d, w = 26, 4, 5
    Q, K, V = rand_unit(rng, L, d)
    st = orc.prefill_statistics(Q, K, V, L, 0.5, recency_window=w, recency_bias=80.0, want_out=True)
    for i in range(L):
        lo = max(0, i - w + 1)
        z = 0.5 * K[lo: i + 1] @ Q[i]
        p = np.exp(z - z.max())
        p /= p.sum()
        assert np.allclose(st.out[i], p @ V[lo: i + 1], rtol=1e-9, atol=1e-12)
    # decode: positions come from pos[], not from the slot index
    res = orc.prefill_compress(Q[:20], K[:20], V[:20], 20, 8, 3, 0.5, recency_window=w, recency_bias=80.0)
    cache = res.cache
    r = orc.decode_step(cache, Q[20], K[20], V[20], 20, 3, 0.5, recency_window=w, recency_bias=80.0)
    near = [j for j in range(cache.n_used) if 0 <= 20 - cache.pos[j] < w]
    assert math.isclose(sum(r.probs[j] for j in near), 1.0, rel_tol=1e-12)
    assert 20 in cache.pos.tolist()


def test_recency_bias_value_enters_the_scaled_logit_additively():
    """Two keys, equal dot products: odds between them are exactly exp(bias)."""
    Q = np.array([[1.0, 0.0]] * 4)
    K = np.array([[0.3, 1.0]] * 4)
    V = np.eye(4)[:, :2]
    st = list(orc.causal_probability_rows(Q, K, 4, 0.25, recency_window=2, recency_bias=0.5))
    P = st[0][1]
    assert math.isclose(P[3, 3] / P[3, 0], math.exp(0.5), rel_tol=1e-12)
    assert math.isclose(P[3, 2] / P[3, 1], math.exp(0.5), rel_tol=1e-12)
    assert math.isclose(P[3, 0], P[3, 1], rel_tol=1e-12)


# ---------------------------------------------------------------------------- selection

def brute_k_smallest(values, k):
    return sorted(i for _, i in sorted((v, i) for i, v in enumerate(values))[:k])


def test_k_smallest_breaks_ties_by_lowest_index():
    rng = np.random.default_rng(8)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        vals = rng.integers(0, 4, n).astype(float)  # many ties
        k = int(rng.integers(1, n + 1))
        assert orc.k_smallest(vals, k).tolist() == brute_k_smallest(vals.tolist(), k)


def test_select_victim_is_scope_then_argmin_with_lowest_index_ties():
    mas = np.array([0.5, 0.1, 0.3, 0.1, 0.05])
    var = np.array([0.0, 2.0, 1.0, 1.0, 9.0])
    assert orc.select_victim(mas, var, 1) == 0  # only the lowest-variance token is in scope
    assert orc.select_victim(mas, var, 2) == 2  # scope {0,2}: tie in variance goes to index 2 first
    assert orc.select_victim(mas, var, 3) == 3  # scope {0,2,3}
    assert orc.select_victim(mas, var, 4) == 1  # scope {0,1,2,3}: equal MAS -> lowest index
    assert orc.select_victim(mas, var, 5) == 4  # everything in scope


def test_closed_form_eviction_set_equals_the_literal_token_by_token_loop():
    rng = np.random.default_rng(9)
    for trial in range(400):
        n = int(rng.integers(2, 14))
        if trial % 2:
            mas, var = rng.random(n), rng.random(n)
        else:  # quantised: plenty of ties in both keys
            mas, var = rng.integers(0, 3, n) / 4.0, rng.integers(0, 3, n) / 4.0
        E = int(rng.integers(1, n))
        s = int(rng.integers(1, n - E + 1))
        assert (orc.select_evictions(mas, var, s, E).tolist()
                == orc.select_evictions_literal(mas, var, s, E).tolist()), (mas, var, s, E)


def test_exhaustive_tiny_selection_against_definition():
    """n = 4, all value patterns from a 2-level alphabet: victim by explicit sort on (key, index)."""
    for mas in itertools.product([0.25, 0.75], repeat=4):
        for var in itertools.product([0.0, 1.0], repeat=4):
            for s in range(1, 5):
                scope = brute_k_smallest(var, s)
                want = min(scope, key=lambda i: (mas[i], i))
                assert orc.select_victim(np.array(mas), np.array(var), s) == want


def test_variance_formula_against_direct_population_variance():
    rng = np.random.default_rng(10)
    for _ in range(20):
        c = int(rng.integers(1, 30))
        x = rng.random(c)
        var = orc.attention_variance([x.sum()], [(x * x).sum()], [c])[0]
        assert math.isclose(var, np.var(x), rel_tol=1e-9, abs_tol=1e-15)  # population, not sample
        assert math.isclose(orc.mean_attention_score([x.sum()], [c])[0], x.mean(), rel_tol=1e-14)
    assert orc.attention_variance([0.3], [0.09], [1])[0] == 0.0  # a single observation


def test_decode_step_is_invariant_to_slot_order():
    rng = np.random.default_rng(11)
    L, d, B, s = 18, 4, 9, 4
    Q, K, V = rand_unit(rng, L + 1, d)
    res = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, 0.6)
    a = res.cache.copy()
    perm = rng.permutation(B)
    b = orc.CacheState(a.K[perm].copy(), a.V[perm].copy(), a.acc[perm].copy(), a.acc2[perm].copy(),
                       a.count[perm].copy(), a.pos[perm].copy(), a.n_used)
    ra = orc.decode_step(a, Q[L], K[L], V[L], L, s, 0.6)
    rb = orc.decode_step(b, Q[L], K[L], V[L], L, s, 0.6)
    assert ra.evicted_pos == rb.evicted_pos and perm[rb.evicted_slot] == ra.evicted_slot
    assert np.allclose(ra.out, rb.out, rtol=1e-12, atol=1e-14)
    oa, ob = np.argsort(a.pos), np.argsort(b.pos)
    assert np.array_equal(a.pos[oa], b.pos[ob])
    assert np.allclose(a.acc[oa], b.acc[ob], rtol=1e-12)
    assert np.allclose(a.acc2[oa], b.acc2[ob], rtol=1e-12)


def test_statistics_memory_is_three_arrays_of_budget_size():
    """Section 5.3 'Overhead': L x H x B x 3 extra elements."""
    rng = np.random.default_rng(12)
    Q, K, V = rand_unit(rng, 12, 4)
    c = orc.prefill_compress(Q, K, V, 12, 5, 2, 0.5).cache
    assert c.acc.shape == c.acc2.shape == c.count.shape == (5,)
    assert c.K.shape == c.V.shape == (5, 4)


def test_heavy_keys_dominate_the_retained_set():
    """Qualitative (not parity): the +4u keys of the workload generator survive compression."""
    from inputs import CONFIGS, make_unit
    cfg = CONFIGS[0]
    u = make_unit(cfg, 0, 0, 0)
    L = cfg.prompt_len
    res = orc.prefill_compress(u.Q[:L], u.K[:L], u.V[:L], L, cfg.budget, cfg.scope, 1 / math.sqrt(cfg.head_dim))
    heavy = [p for p in u.heavy_positions if p < L]
    kept = sum(1 for p in heavy if p in set(res.retained.tolist()))
    assert kept >= 0.8 * len(heavy)


# ---------------------------------------------------------------------------- block-wise evict-and-encode

def test_block_of_one_is_exactly_a_decode_step():
    rng = np.random.default_rng(21)
    L, d, B, s = 30, 5, 12, 4
    Q, K, V = rand_unit(rng, L + 6, d)
    a = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, 0.4).cache
    b = a.copy()
    for t in range(L, L + 6):
        ra = orc.decode_step(a, Q[t], K[t], V[t], t, s, 0.4)
        rb = orc.encode_block(b, Q[t:t + 1], K[t:t + 1], V[t:t + 1], t, s, 0.4)
        assert np.array_equal(ra.out, rb.out[0]) and ra.evicted_slot == rb.evicted_slot[0]
        assert ra.evicted_pos == rb.evicted_pos[0]
        for x, y in ((a.acc, b.acc), (a.acc2, b.acc2), (a.count, b.count), (a.pos, b.pos), (a.K, b.K)):
            assert np.array_equal(x, y)


@pytest.mark.parametrize("b", [1, 2, 3, 7])
def test_blocks_without_eviction_reproduce_dense_causal_attention(b):
    """Budget >= total length: block-wise encoding of a whole sequence equals textbook causal attention."""
    rng = np.random.default_rng(22 + b)
    T, d = 23, 4
    Q, K, V = rand_unit(rng, T, d)
    P, O = dense_causal_attention(Q, K, V, 0.6)
    st = orc.CacheState(np.zeros((T + 3, d)), np.zeros((T + 3, d)), np.zeros(T + 3), np.zeros(T + 3),
                        np.zeros(T + 3), np.full(T + 3, -1, dtype=np.int64), 0)
    t = 0
    while t < T:
        bb = min(b, T - t)
        r = orc.encode_block(st, Q[t:t + bb], K[t:t + bb], V[t:t + bb], t, 3, 0.6)
        assert np.allclose(r.out, O[t:t + bb], rtol=1e-12, atol=1e-14)
        assert np.all(r.evicted_slot == -1) and r.slots.tolist() == list(range(t, t + bb))
        t += bb
    assert st.n_used == T and np.array_equal(st.pos[:T], np.arange(T))
    assert np.allclose(st.acc[:T], P.sum(0), rtol=1e-12)
    assert np.allclose(st.acc2[:T], (P ** 2).sum(0), rtol=1e-12)
    assert np.array_equal(st.count[:T], T - np.arange(T))


@pytest.mark.parametrize("b", [2, 4, 5])
def test_blockwise_eviction_keeps_the_budget_and_its_statistics_equal_a_brute_force_recount(b):
    rng = np.random.default_rng(30 + b)
    T, d, B, s = 41, 4, 9, 3
    Q, K, V = rand_unit(rng, T, d)
    st = orc.CacheState(np.zeros((B, d)), np.zeros((B, d)), np.zeros(B), np.zeros(B), np.zeros(B),
                        np.full(B, -1, dtype=np.int64), 0)
    log = []  # (query position, {key position: probability})
    t = 0
    while t < T:
        bb = min(b, T - t)
        before_pos, before_n = st.pos.copy(), st.n_used
        if before_n + bb > B:
            mas = orc.mean_attention_score(st.acc[:before_n], st.count[:before_n])
            var = orc.attention_variance(st.acc[:before_n], st.acc2[:before_n], st.count[:before_n])
            want = orc.select_evictions_literal(mas, var, s, before_n + bb - B)  # the token-by-token loop
        else:
            want = np.zeros(0, dtype=np.int64)
        r = orc.encode_block(st, Q[t:t + bb], K[t:t + bb], V[t:t + bb], t, s, 0.5)
        assert st.n_used <= B
        assert sorted(x for x in r.evicted_slot.tolist() if x >= 0) == want.tolist()
        for i in range(bb):
            assert st.pos[r.slots[i]] == t + i
            if r.evicted_slot[i] >= 0:
                assert r.evicted_pos[i] == before_pos[r.evicted_slot[i]]
            row = {int(st.pos[j]): r.probs[i][j] for j in range(st.n_used) if r.probs[i][j] > 0}
            assert abs(sum(row.values()) - 1.0) < 1e-12
            assert max(row) == t + i and all(p <= t + i for p in row)  # causal inside the block
            log.append((t + i, row))
            z = np.array([0.5 * np.dot(Q[t + i], K[p]) for p in row])
            w = np.exp(z - z.max())
            w /= w.sum()
            assert np.allclose(r.out[i], sum(wi * V[p] for wi, p in zip(w, row)), rtol=1e-12, atol=1e-14)
        t += bb
    for j in range(st.n_used):
        p = int(st.pos[j])
        rows = [row[p] for (_, row) in log if p in row]
        assert st.count[j] == len(rows)
        assert math.isclose(st.acc[j], math.fsum(rows), rel_tol=1e-12)
        assert math.isclose(st.acc2[j], math.fsum(x * x for x in rows), rel_tol=1e-12)


# ---------------------------------------------------------------------------- grouped-query attention

def test_group_of_one_is_exactly_a_decode_step_and_identical_heads_change_nothing():
    rng = np.random.default_rng(41)
    L, d, B, s = 26, 4, 10, 3
    Q, K, V = rand_unit(rng, L + 5, d)
    a = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, 0.5).cache
    b, c = a.copy(), a.copy()
    for t in range(L, L + 5):
        ra = orc.decode_step(a, Q[t], K[t], V[t], t, s, 0.5)
        rb = orc.decode_step_gqa(b, Q[t:t + 1], K[t], V[t], t, s, 0.5)
        rc = orc.decode_step_gqa(c, np.stack([Q[t]] * 3), K[t], V[t], t, s, 0.5)
        assert np.array_equal(ra.out, rb.out[0]) and ra.evicted_slot == rb.evicted_slot == rc.evicted_slot
        assert np.allclose(rc.out, ra.out[None], rtol=1e-13)
        for x, y, z in ((a.acc, b.acc, c.acc), (a.acc2, b.acc2, c.acc2), (a.count, b.count, c.count)):
            assert np.array_equal(x, y) and np.allclose(x, z, rtol=1e-13)


def test_group_statistics_receive_the_mean_of_independently_computed_softmaxes():
    rng = np.random.default_rng(42)
    L, d, B, s, g = 18, 5, 18, 4, 4
    Q, K, V = rand_unit(rng, L, d)
    st = orc.prefill_compress(Q, K, V, L, B + 1, s, 0.3).cache  # one free slot: the step appends
    Qg = rng.standard_normal((g, d))
    kn, vn = rng.standard_normal(d), rng.standard_normal(d)
    acc0, acc20, cnt0 = st.acc.copy(), st.acc2.copy(), st.count.copy()
    r = orc.decode_step_gqa(st, Qg, kn, vn, L, s, 0.3)
    keys = np.vstack([K, kn])
    vals = np.vstack([V, vn])
    rows = []
    for h in range(g):
        z = 0.3 * keys @ Qg[h]
        w = np.exp(z - z.max())
        w /= w.sum()
        rows.append(w)
        assert np.allclose(r.out[h], w @ vals, rtol=1e-12)
    mean = np.mean(rows, axis=0)
    assert np.allclose(r.mean_probs, mean, rtol=1e-12) and abs(mean.sum() - 1.0) < 1e-12
    assert np.allclose(st.acc[:L + 1], np.append(acc0[:L], 0.0) + mean, rtol=1e-12)
    assert np.allclose(st.acc2[:L + 1], np.append(acc20[:L], 0.0) + mean ** 2, rtol=1e-12)
    assert np.array_equal(st.count[:L + 1], np.append(cnt0[:L], 0.0) + 1.0)  # one count per step, not per head


def test_grouped_block_reduces_to_the_block_step_and_to_the_grouped_decode_step():
    rng = np.random.default_rng(43)
    L, d, B, s = 30, 4, 12, 3
    Q, K, V = rand_unit(rng, L + 12, d)
    a = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, 0.5).cache
    b_, c, e = a.copy(), a.copy(), a.copy()
    t = L
    for blk in (3, 1, 5):  # one head per group: the block-wise step
        ra = orc.encode_block(a, Q[t:t + blk], K[t:t + blk], V[t:t + blk], t, s, 0.5, 3, 0.25)
        rb = orc.encode_block_gqa(b_, Q[t:t + blk, None], K[t:t + blk], V[t:t + blk], t, s, 0.5, 3, 0.25)
        assert np.array_equal(ra.out, rb.out[:, 0]) and np.array_equal(ra.evicted_slot, rb.evicted_slot)
        for x, y in ((a.acc, b_.acc), (a.acc2, b_.acc2), (a.count, b_.count), (a.pos, b_.pos)):
            assert np.array_equal(x, y)
        t += blk
    for t in range(L, L + 4):  # one token per block: the grouped decode step
        Qg = rng.standard_normal((3, d))
        rc = orc.decode_step_gqa(c, Qg, K[t], V[t], t, s, 0.5, 3, 0.25)
        re = orc.encode_block_gqa(e, Qg[None], K[t:t + 1], V[t:t + 1], t, s, 0.5, 3, 0.25)
        assert np.array_equal(rc.out, re.out[0]) and rc.evicted_slot == int(re.evicted_slot[0])
        for x, y in ((c.acc, e.acc), (c.acc2, e.acc2), (c.count, e.count), (c.pos, e.pos)):
            assert np.array_equal(x, y)


def test_grouped_blocks_without_eviction_accumulate_the_head_mean_of_dense_causal_attention():
    rng = np.random.default_rng(44)
    L, d, g = 13, 5, 3
    Qh = rng.standard_normal((g, L, d))
    _, K, V = rand_unit(rng, L, d)
    st = orc.CacheState(np.zeros((L, d)), np.zeros((L, d)), np.zeros(L), np.zeros(L), np.zeros(L),
                        np.full(L, -1, dtype=np.int64), 0)
    t, outs = 0, []
    for blk in (4, 1, 6, 2):
        r = orc.encode_block_gqa(st, Qh[:, t:t + blk].transpose(1, 0, 2), K[t:t + blk], V[t:t + blk], t, 2, 0.4)
        outs.append(r.out)
        t += blk
    Z = 0.4 * np.einsum("hid,jd->hij", Qh, K)  # dense causal softmax per head, written out here
    Z = np.where(np.tril(np.ones((L, L), dtype=bool))[None], Z, -np.inf)
    P = np.exp(Z - Z.max(axis=2, keepdims=True))
    P /= P.sum(axis=2, keepdims=True)
    mean = P.mean(axis=0)
    assert np.allclose(st.acc, mean.sum(axis=0), rtol=1e-12)
    assert np.allclose(st.acc2, (mean ** 2).sum(axis=0), rtol=1e-12)
    assert np.array_equal(st.count, L - np.arange(L))
    out = np.concatenate(outs)  # [L, g, d]
    for h in range(g):
        assert np.allclose(out[:, h], P[h] @ V, rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------------------- other policies of the same framework

def test_recency_policy_with_sinks_is_the_sliding_window_with_attention_sinks_in_closed_form():
    """importance "oldest" over the whole cache with k protected first positions: after any number of steps the
    cache holds positions 0..k-1 and the most recent B-k ones, and each output is dense softmax attention over
    exactly that set (computed here from the full K / V, with no cache)."""
    rng = np.random.default_rng(51)
    L, T, d, B, k = 20, 15, 4, 9, 3
    Q, K, V = rand_unit(rng, L + T, d)
    pol = orc.Policy("oldest", "all", k)
    r = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, 1, 0.5, policy=pol)
    st = r.cache
    assert list(st.pos) == list(range(k)) + list(range(L - (B - k), L))
    for t in range(L, L + T):
        res = orc.decode_step(st, Q[t], K[t], V[t], t, 1, 0.5, policy=pol)
        keep = list(range(k)) + list(range(t - (B - k) + 1, t + 1))
        assert sorted(st.pos) == keep and res.evicted_pos == t - (B - k)
        z = 0.5 * K[keep] @ Q[t]
        w = np.exp(z - z.max())
        w /= w.sum()
        assert np.allclose(res.out, w @ V[keep], rtol=1e-12)


def test_accumulated_score_policy_evicts_the_argmin_of_an_independent_recount():
    """importance "aas" over the whole cache (the accumulated attention score of section 4.1): the evicted
    position is the argmin of sums rebuilt from a log of every attention row."""
    rng = np.random.default_rng(52)
    L, T, d, B = 16, 20, 5, 16
    Q, K, V = rand_unit(rng, L + T, d)
    pol = orc.Policy("aas", "all")
    r = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, 3, 0.4, policy=pol)
    st = r.cache
    total = {int(p): float(a) for p, a in zip(st.pos, st.acc)}  # B = L: nothing evicted yet, Acc = column sums
    dense = np.zeros(L)
    for i in range(L):
        z = 0.4 * K[:i + 1] @ Q[i]
        w = np.exp(z - z.max())
        dense[:i + 1] += w / w.sum()
    assert np.allclose([total[j] for j in range(L)], dense, rtol=1e-12)
    for t in range(L, L + T):
        expect = min(total, key=lambda j: (total[j], j))
        res = orc.decode_step(st, Q[t], K[t], V[t], t, 3, 0.4, policy=pol)
        assert res.evicted_pos == expect
        del total[expect]
        total[t] = 0.0
        for slot in range(B):
            total[int(st.pos[slot])] += float(res.probs[slot])


def test_window_scope_protects_the_most_recent_tokens_and_picks_by_explicit_sort():
    rng = np.random.default_rng(53)
    L, T, d, B, s = 30, 25, 4, 12, 5
    Q, K, V = rand_unit(rng, L + T, d)
    for imp in ("mas", "aas"):
        pol = orc.Policy(imp, "window")
        st = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, 0.5, policy=pol).cache
        for t in range(L, L + T):
            before = st.copy()
            res = orc.decode_step(st, Q[t], K[t], V[t], t, s, 0.5, policy=pol)
            oldest = sorted(range(B), key=lambda j: before.pos[j])[:s]
            score = before.acc / before.count if imp == "mas" else before.acc
            expect = min(oldest, key=lambda j: (score[j], j))
            assert res.evicted_slot == expect
            assert res.evicted_pos not in sorted(before.pos)[s:]  # the B - s most recent are never touched


def test_default_policy_is_roco_and_block_steps_accept_a_policy():
    rng = np.random.default_rng(54)
    L, d, B, s = 24, 4, 10, 3
    Q, K, V = rand_unit(rng, L + 6, d)
    a = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, 0.5).cache
    b = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, 0.5, policy=orc.Policy("mas", "std")).cache
    assert np.array_equal(a.pos, b.pos) and np.array_equal(a.acc, b.acc)
    pol = orc.Policy("oldest", "all", 2)
    c = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, s, 0.5, policy=pol).cache
    e = c.copy()
    for t in range(L, L + 6):
        orc.decode_step(c, Q[t], K[t], V[t], t, s, 0.5, policy=pol)
    orc.encode_block(e, Q[L:L + 6], K[L:L + 6], V[L:L + 6], L, s, 0.5, policy=pol)
    assert sorted(c.pos) == sorted(e.pos) == [0, 1] + list(range(L + 6 - 8, L + 6))


def test_shrinking_a_dense_cache_keeps_what_prefill_compress_keeps():
    rng = np.random.default_rng(61)
    L, d, s = 40, 4, 6
    Q, K, V = rand_unit(rng, L, d)
    for pol in (None, orc.Policy("aas", "all"), orc.Policy("mas", "window"), orc.Policy("oldest", "all", 3)):
        dense = orc.prefill_compress(Q, K, V, L, L + 5, s, 0.5, policy=pol).cache
        for keep in (1, 13, 39, 40, 60):
            mask = orc.select_retained(dense, keep, s, pol)
            want = orc.prefill_compress(Q, K, V, L, keep, s, 0.5, policy=pol).retained
            assert np.array_equal(dense.pos[mask], want) and mask.sum() == min(keep, L)
        assert not mask[L:].any()  # empty slots are never reported


def test_last_token_score_keeps_the_top_of_the_last_query_row_written_out_independently():
    """importance "ltas" over the whole cache (section 4.1, the score of TOVA): after the prompt the cache holds
    the B tokens with the highest attention from the last prompt token, and every decode step evicts the cached
    token the previous query attended least; both are rebuilt here from dense softmax rows, without the cache."""
    rng = np.random.default_rng(71)
    L, T, d, B = 24, 12, 5, 9
    Q, K, V = rand_unit(rng, L + T, d)
    pol = orc.Policy("ltas", "all")
    r = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, 1, 0.45, policy=pol)
    z = 0.45 * K[:L] @ Q[L - 1]
    w = np.exp(z - z.max())
    w /= w.sum()
    assert np.allclose(r.full.acc2, w, rtol=1e-12)
    assert sorted(r.retained) == sorted(np.argsort(-w, kind="stable")[:B])
    st = r.cache
    held = {int(p): float(x) for p, x in zip(st.pos, st.acc2)}  # position -> score from the latest query
    for t in range(L, L + T):
        expect = min(held, key=lambda j: (held[j], list(st.pos).index(j)))
        res = orc.decode_step(st, Q[t], K[t], V[t], t, 1, 0.45, policy=pol)
        assert res.evicted_pos == expect
        keep = [int(p) for p in st.pos]
        zz = 0.45 * K[keep] @ Q[t]
        ww = np.exp(zz - zz.max())
        ww /= ww.sum()
        held = dict(zip(keep, ww))
        assert np.allclose(st.acc2, ww, rtol=1e-12) and np.allclose(res.out, ww @ V[keep], rtol=1e-12)
    with pytest.raises(ValueError):
        orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, 3, 0.45, policy=orc.Policy("ltas", "std"))


def test_last_token_score_in_block_and_grouped_steps_is_the_last_tokens_row():
    rng = np.random.default_rng(72)
    L, d, B = 20, 4, 12
    Q, K, V = rand_unit(rng, L + 5, d)
    pol = orc.Policy("ltas", "window")
    a = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, 6, 0.5, policy=pol).cache
    b = a.copy()
    r = orc.encode_block(a, Q[L:L + 5], K[L:L + 5], V[L:L + 5], L, 6, 0.5, policy=pol)
    assert np.array_equal(a.acc2, r.probs[4])  # every slot is seen by the block's last token
    Qg = np.stack([Q[L:L + 5], Q[L:L + 5][::-1]], axis=1)  # two heads
    rg = orc.encode_block_gqa(b, Qg, K[L:L + 5], V[L:L + 5], L, 6, 0.5, policy=pol)
    assert np.array_equal(b.acc2, rg.mean_probs[4]) and np.array_equal(a.pos, b.pos)


def test_grouped_prefill_statistics_reduce_to_one_head_and_equal_block_wise_encoding_without_eviction():
    rng = np.random.default_rng(81)
    L, d, g = 23, 4, 3
    Qh = rng.standard_normal((g, L, d))
    _, K, V = rand_unit(rng, L, d)
    one = orc.prefill_statistics_gqa(Qh[:1], K, V, L, 0.5, 4, 0.3, row_block=7)
    ref = orc.prefill_statistics(Qh[0], K, V, L, 0.5, 4, 0.3)
    assert np.allclose(one.acc, ref.acc, rtol=1e-13) and np.allclose(one.acc2, ref.acc2, rtol=1e-13)
    assert np.array_equal(one.count, ref.count)
    full = orc.prefill_statistics_gqa(Qh, K, V, L, 0.5, 4, 0.3, row_block=7)
    st = orc.CacheState(np.zeros((L, d)), np.zeros((L, d)), np.zeros(L), np.zeros(L), np.zeros(L),
                        np.full(L, -1, dtype=np.int64), 0)
    t = 0
    for blk in (5, 1, 9, 8):  # the same prompt, encoded block-wise into a cache that never fills
        orc.encode_block_gqa(st, Qh[:, t:t + blk].transpose(1, 0, 2), K[t:t + blk], V[t:t + blk], t, 3, 0.5, 4, 0.3)
        t += blk
    assert np.allclose(full.acc, st.acc, rtol=1e-12) and np.allclose(full.acc2, st.acc2, rtol=1e-12)
    assert np.array_equal(full.count, st.count)
    # the last-token score: the head-mean of the last prompt token's rows
    last = orc.prefill_statistics_gqa(Qh, K, V, L, 0.5, policy=orc.Policy("ltas", "all"))
    rows = []
    for h in range(g):
        z = 0.5 * K @ Qh[h, L - 1]
        w = np.exp(z - z.max())
        rows.append(w / w.sum())
    assert np.allclose(last.acc2, np.mean(rows, axis=0), rtol=1e-12)
    r = orc.prefill_compress_gqa(Qh, K, V, L, 10, 4, 0.5)
    assert r.cache.n_used == 10 and np.array_equal(r.cache.acc, full_acc_at(r, orc.prefill_statistics_gqa(Qh, K, V, L, 0.5)))


def full_acc_at(result, full):
    return np.concatenate([full.acc[result.retained], np.zeros(result.cache.budget - result.retained.shape[0])])


def test_quantised_score_equals_an_explicit_recount_of_above_average_attention():
    """importance "aqas" (section 4.1: the attention score quantised to 1 above / 0 below the row average): the
    second array equals a count rebuilt from dense attention rows with plain loops, and each eviction takes the
    argmin of that count (ties: lowest slot)."""
    rng = np.random.default_rng(91)
    L, T, d, B = 14, 18, 5, 14
    Q, K, V = rand_unit(rng, L + T, d)
    pol = orc.Policy("aqas", "all")
    st = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, 3, 0.6, policy=pol).cache  # B = L: nothing evicted yet
    count = {}
    for j in range(L):
        c = 0
        for i in range(j, L):
            z = 0.6 * K[:i + 1] @ Q[i]
            w = np.exp(z - z.max())
            w /= w.sum()
            c += 1 if w[j] > 1.0 / (i + 1) else 0
        count[j] = c
    assert [count[int(p)] for p in st.pos] == list(st.acc2)
    assert max(st.acc2) >= 2 and min(st.acc2) == 0  # the case is not degenerate
    for t in range(L, L + T):
        slots = list(st.pos)
        expect = min(range(B), key=lambda sl: (count[int(slots[sl])], sl))
        res = orc.decode_step(st, Q[t], K[t], V[t], t, 3, 0.6, policy=pol)
        assert res.evicted_slot == expect
        del count[res.evicted_pos]
        count[t] = 0
        keep = [int(p) for p in st.pos]
        z = 0.6 * K[keep] @ Q[t]
        w = np.exp(z - z.max())
        w /= w.sum()
        for sl, p in enumerate(keep):
            count[p] += 1 if w[sl] > 1.0 / B else 0
        assert [count[p] for p in keep] == list(st.acc2)


def test_row_normalisers_closed_forms():
    """Q = 0: every visible logit is 0, so lse[i] = ln(i + 1).  d = 1, q = 1, k = ln w, scale 1: lse[i] = ln of the
    prefix sum of w.  A recency bias b on the last w positions multiplies their terms by e^b."""
    L, d = 37, 8
    rng = np.random.default_rng(5)
    K = rng.standard_normal((L, d))
    assert np.allclose(orc.row_log_sum_exp(np.zeros((L, d)), K, L, 0.3), np.log(np.arange(1, L + 1)), rtol=0, atol=1e-13)
    w = rng.uniform(0.5, 3.0, size=L)
    got = orc.row_log_sum_exp(np.ones((L, 1)), np.log(w)[:, None], L, 1.0, row_block=7)
    assert np.allclose(got, np.log(np.cumsum(w)), rtol=0, atol=1e-13)
    b, win = 0.5, 4
    want = np.empty(L)
    for i in range(L):
        terms = [w[j] * (math.e ** b if i - j < win else 1.0) for j in range(i + 1)]
        want[i] = math.log(sum(terms))
    got = orc.row_log_sum_exp(np.ones((L, 1)), np.log(w)[:, None], L, 1.0, win, b, row_block=5)
    assert np.allclose(got, want, rtol=0, atol=1e-13)


def test_row_normalisers_give_back_the_probabilities():
    """exp(logit - lse) are the rows of the causal softmax: they sum to one and match the dense definition."""
    L, d = 29, 6
    rng = np.random.default_rng(6)
    Q, K = rng.standard_normal((L, d)), rng.standard_normal((L, d))
    sc = 0.37
    lse = orc.row_log_sum_exp(Q, K, L - 3, sc, 5, 0.25, row_block=8)  # a length shorter than the arrays
    assert lse.shape == (L - 3,)
    for i in range(L - 3):
        logits = np.array([sc * float(Q[i] @ K[j]) + (0.25 if i - j < 5 else 0.0) for j in range(i + 1)])
        p = np.exp(logits - lse[i])
        assert abs(p.sum() - 1.0) < 1e-13


# ---------------------------------------------------------------------------- quantised score in the block / grouped paths

def _softmax_over(K_rows, q, scale):
    """One softmax row written out with plain Python loops (section 2.1, eq. 1)."""
    logits = [scale * sum(float(a) * float(b) for a, b in zip(k, q)) for k in K_rows]
    top = max(logits)
    e = [math.exp(x - top) for x in logits]
    tot = sum(e)
    return [x / tot for x in e]


def _recount_block(st_before, Qb, Kb, Vb, qpos0, slots, scale, heads, wrong_average=False):
    """What the three arrays must hold after a block has been encoded into the slots `slots` (already known: which
    slots a block takes is pinned elsewhere), rebuilt token by token with loops: the block's token i attends the
    older tokens and the block's tokens 0..i; a slot's second array counts the rows whose (head-mean) probability
    for it was above the average of that row, 1 / (number of tokens the row attended) (section 4.1, quantised
    score).  `wrong_average` divides by the cache's final occupancy instead: the mistake the pin must catch."""
    B = st_before.budget
    K = [list(r) for r in st_before.K]
    acc, acc2, cnt = list(st_before.acc), list(st_before.acc2), list(st_before.count)
    in_block = {}
    for i, s in enumerate(slots):
        K[s] = list(Kb[i])
        acc[s] = acc2[s] = cnt[s] = 0.0
        in_block[int(s)] = i
    n_new = min(B, st_before.n_used + len(slots))
    for i in range(len(slots)):
        seen = [s for s in range(n_new) if in_block.get(s, -1) <= i]
        rows = [_softmax_over([K[s] for s in seen], Qb[i][h] if heads else Qb[i], scale) for h in range(heads or 1)]
        mean = [sum(r[t] for r in rows) / len(rows) for t in range(len(seen))]
        avg_of = n_new if wrong_average else len(seen)
        for t, s in enumerate(seen):
            acc[s] += mean[t]
            acc2[s] += 1.0 if mean[t] * avg_of > 1.0 else 0.0
            cnt[s] += 1.0
    return acc, acc2, cnt


def test_quantised_score_in_a_block_counts_against_the_tokens_each_row_attended():
    """encode_block under importance "aqas": a block that straddles a full cache (some tokens take empty slots, some
    take over evicted ones), so the rows of one block attend different numbers of tokens; the count of above-average
    rows is rebuilt with loops over dense softmax rows and compared exactly.  A recount that takes the average over
    the final occupancy instead of over what each row attended gives different numbers on this case."""
    rng = np.random.default_rng(101)
    L, d, B, b = 9, 4, 12, 6
    Q, K, V = rand_unit(rng, L + b, d)
    pol = orc.Policy("aqas", "all")
    st = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, 3, 0.8, policy=pol).cache  # 9 of 12 slots used
    before = st.copy()
    Qb = 0.4 * Q[L:L + b]  # flat rows: many probabilities lie between 1/12 and 1/7, where the two averages differ
    blk = orc.encode_block(st, Qb, K[L:L + b], V[L:L + b], L, 3, 0.8, policy=pol)
    assert (blk.evicted_slot >= 0).sum() == 3 and (blk.evicted_slot < 0).sum() == 3  # straddles the budget
    acc, acc2, cnt = _recount_block(before, Qb, K[L:L + b], V[L:L + b], L, blk.slots, 0.8, heads=0)
    assert list(st.acc2) == acc2 and list(st.count) == cnt
    assert np.allclose(st.acc, acc, rtol=1e-12)
    _, wrong, _ = _recount_block(before, Qb, K[L:L + b], V[L:L + b], L, blk.slots, 0.8, heads=0, wrong_average=True)
    assert wrong != acc2  # the case tells the two averages apart


def test_quantised_score_in_a_grouped_block_thresholds_the_head_mean():
    """encode_block_gqa under "aqas": the head-mean probability of each of the block's tokens is compared with the
    average of that token's row; loops over dense per-head softmax rows, exact comparison, same straddling block."""
    rng = np.random.default_rng(102)
    L, d, B, b, g = 10, 4, 13, 5, 3
    Q, K, V = rand_unit(rng, L + b, d)
    Qg = rng.standard_normal((b, g, d)) * 0.5  # flat rows, see the ungrouped test
    pol = orc.Policy("aqas", "window")
    st = orc.prefill_compress(Q[:L], K[:L], V[:L], L, B, 4, 0.7, policy=pol).cache  # 10 of 13 slots used
    before = st.copy()
    blk = orc.encode_block_gqa(st, Qg, K[L:L + b], V[L:L + b], L, 4, 0.7, policy=pol)
    assert (blk.evicted_slot >= 0).sum() == 2 and (blk.evicted_slot < 0).sum() == 3
    acc, acc2, cnt = _recount_block(before, Qg, K[L:L + b], V[L:L + b], L, blk.slots, 0.7, heads=g)
    assert list(st.acc2) == acc2 and list(st.count) == cnt
    assert np.allclose(st.acc, acc, rtol=1e-12)
    _, wrong, _ = _recount_block(before, Qg, K[L:L + b], V[L:L + b], L, blk.slots, 0.7, heads=g, wrong_average=True)
    assert wrong != acc2
    # thresholding each head and averaging the bits is a different statistic; the case tells them apart too
    per_head = [0.0] * B
    in_block = {int(s): i for i, s in enumerate(blk.slots)}
    Kn = [list(r) for r in st.K]
    for i in range(b):
        seen = [s for s in range(st.n_used) if in_block.get(s, -1) <= i]
        for h in range(g):
            row = _softmax_over([Kn[s] for s in seen], Qg[i][h], 0.7)
            for t, s in enumerate(seen):
                per_head[s] += (1.0 if row[t] * len(seen) > 1.0 else 0.0) / g
    base = [0.0 if int(s) in in_block else float(before.acc2[s]) for s in range(B)]
    assert [x + y for x, y in zip(base, per_head)] != acc2


def test_grouped_prefill_quantised_score_and_outputs_from_dense_per_head_softmaxes():
    """prefill_statistics_gqa: (1) under "aqas" the second array counts the rows i whose head-mean probability for
    key j exceeds 1 / (i + 1); (2) want_out returns every head's own P_h V.  Both against dense causal attention
    written separately (einsum softmax per head)."""
    rng = np.random.default_rng(103)
    L, d, g = 19, 5, 4
    Qh = rng.standard_normal((g, L, d)) * 1.3
    _, K, V = rand_unit(rng, L, d)
    sc = 0.6
    Ps, Os = zip(*(dense_causal_attention(Qh[h], K, V, sc) for h in range(g)))
    Pbar = sum(Ps) / g
    want = [sum(1.0 for i in range(j, L) if Pbar[i, j] > 1.0 / (i + 1)) for j in range(L)]
    got = orc.prefill_statistics_gqa(Qh, K, V, L, sc, row_block=6, policy=orc.Policy("aqas", "all"), want_out=True)
    assert list(got.acc2) == want
    assert max(want) >= 3 and min(want) == 0  # not degenerate
    assert np.allclose(got.acc, Pbar.sum(0), rtol=1e-12)
    assert np.array_equal(got.count, L - np.arange(L))
    assert got.out.shape == (g, L, d)
    for h in range(g):
        assert np.allclose(got.out[h], Os[h], rtol=1e-12, atol=1e-14)
    # each head's output is its own, not the head-mean's: swapping two heads swaps the outputs
    swapped = orc.prefill_statistics_gqa(Qh[[1, 0, 2, 3]], K, V, L, sc, want_out=True)
    assert np.allclose(swapped.out[0], Os[1], rtol=1e-12) and np.allclose(swapped.out[1], Os[0], rtol=1e-12)
    assert np.allclose(swapped.acc2, (Pbar ** 2).sum(0), rtol=1e-12)  # default policy: squares of the head-mean
    # thresholding per head and averaging the bits is a different statistic
    bits = sum((P * np.arange(1, L + 1)[:, None] > 1.0) & np.tril(np.ones((L, L), bool)) for P in Ps) / g
    assert list(bits.sum(0)) != want
