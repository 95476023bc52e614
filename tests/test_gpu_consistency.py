"""GPU parity of roco_select_retained and of the synthetic consistency study (section 4.1, Fig. 2) with the
same study run on the oracle."""
import math

import numpy as np
import pytest
import torch

from inputs import round_to_bf16
from oracle import roco_oracle as orc

pytestmark = pytest.mark.gpu


def _P():
    import parity
    return parity


def _data(units, T, d, seed):
    rng = np.random.default_rng(seed)
    Q = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32) + 0.25)
    K = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    heavy = rng.choice(T, size=max(1, T // 25), replace=False)
    u = rng.standard_normal(d).astype(np.float32)
    K[:, heavy] = round_to_bf16(K[:, heavy] + 3 * u / np.linalg.norm(u))
    return Q, K, V


@pytest.mark.parametrize("pol", [orc.ROCO, orc.Policy("aas", "all"), orc.Policy("mas", "window"),
                                 orc.Policy("oldest", "all", 3)], ids=["roco", "aas-all", "mas-window", "sinks"])
def test_select_retained_matches_the_oracle(pol):
    import paper_2402_06262_amd as roco
    P = _P()
    units, d, B, s = 4, 128, 160, 40
    lens = [160, 150, 90, 7]
    Q, K, V = _data(units, 160, d, 11)
    sess = P.make_session(units, d, B, s, "bf16", policy=pol)
    g = P.gpu_prefill(sess, Q, K, V, lens, False)
    states = [P.check_prefill_unit(g, u, Q[u], K[u], V[u], lens[u], B, s, 1 / math.sqrt(d), "bf16", 0, 0.0, False,
                                   policy=pol)[0].cache for u in range(units)]
    c = sess.cache
    for keep in (0, 1, 33, 89, 90, 159, 160, 500):
        mask = torch.full((units, B), -5, dtype=torch.int32, device="cuda")
        roco.roco_select_retained(sess.params, keep, c.stats, c.pos, c.n_used, mask, sess.decode_ws)
        torch.cuda.synchronize()
        got = mask.cpu().numpy()
        for u in range(units):
            want = orc.select_retained(states[u], keep, s, pol)
            if not np.array_equal(got[u].astype(bool), want):  # only a declared tie may differ
                st = states[u]
                n = st.n_used
                imp, key, s_eff = orc.ranking_scores(pol, st.acc[:n], st.acc2[:n], st.count[:n], st.pos[:n], s)
                from oracle import tie_band
                eps_m, eps_v = tie_band.bands_for(pol, st.acc[:n], st.acc2[:n], st.count[:n])
                ok, why = tie_band.admissible_eviction(imp, key, eps_m, eps_v, s_eff, n - keep,
                                                       np.flatnonzero(~got[u, :n].astype(bool)))
                assert ok, f"keep {keep} unit {u}: {why}"
            assert set(np.unique(got[u])) <= {0, 1} and got[u].sum() == min(keep, lens[u])


def test_consistency_study_matches_the_same_study_on_the_oracle():
    from paper_2402_06262_amd.consistency import consistency_study
    units, d, L, T = 3, 128, 48, 112
    rates = (0.3, 0.5)
    Q, K, V = _data(units, T, d, 23)
    dev = [torch.from_numpy(x).cuda().to(torch.bfloat16) for x in (Q, K, V)]
    raw = {}
    got = consistency_study(*dev, prompt_len=L, rates=rates, importances=("mas", "aas", "oldest", "ltas", "aqas"), sample_every=4,
                            counts=raw)
    compared = differing = 0
    sc = 1 / math.sqrt(d)
    sampled = [t for t in range(L, T) if (t - L) % 4 == 3 or t == T - 1]
    for name in ("mas", "aas", "oldest", "ltas", "aqas"):
        pol = orc.Policy(name, "all")
        for r in rates:
            B = int(round(r * T))
            tot, cnt = 0.0, 0
            for u in range(units):
                full = orc.prefill_compress(Q[u, :L], K[u, :L], V[u, :L], L, T, T, sc, policy=pol).cache
                small = orc.prefill_compress(Q[u, :L], K[u, :L], V[u, :L], L, B, B, sc, policy=pol).cache
                for t in range(L, T):
                    orc.decode_step(full, Q[u, t], K[u, t], V[u, t], t, T, sc, policy=pol)
                    orc.decode_step(small, Q[u, t], K[u, t], V[u, t], t, B, sc, policy=pol)
                    if t in sampled and t + 1 > B:
                        top = set(full.pos[orc.select_retained(full, B, T, pol)].tolist())
                        held = set(small.pos[:small.n_used].tolist())
                        tot += len(top & held) / len(top | held)
                        cnt += 1
                        # position by position and unit by unit: the same two set sizes, except where an fp32 / fp64
                        # near-tie swapped a member of one of the sets (each swap moves a size by at most one)
                        gi, gu = (int(x[u]) for x in raw[(name, r, t)])
                        compared += 1
                        if (gi, gu) != (len(top & held), len(top | held)):
                            differing += 1
                            assert abs(gi - len(top & held)) <= 2 and abs(gu - len(top | held)) <= 2, (name, r, t, u)
            mean, n = got[name][r]
            print(f"{name} rate {r}: library {mean:.4f} oracle {tot / cnt:.4f} over {cnt} positions", flush=True)
            assert n == cnt
            assert abs(mean - tot / cnt) < 5e-3  # identical sets up to fp32 / fp64 near-ties in a few positions
    print(f"set sizes compared per position and unit: {compared}, differing by a swapped member: {differing}", flush=True)
    assert differing <= 0.05 * compared
    # closed form: recency is perfectly consistent with its own full-cache variant (both are the last B tokens)
    assert got["oldest"][0.3][0] == 1.0 and got["oldest"][0.5][0] == 1.0


def test_set_overlap_counts_against_python_sets():
    """roco_set_overlap on random caches: masked and unmasked sets, partially filled units, an empty set."""
    import paper_2402_06262_amd as roco
    rng = np.random.default_rng(5)
    units, sa, sb, T = 5, 96, 40, 300
    pos_a = np.stack([rng.choice(T, size=sa, replace=False) for _ in range(units)]).astype(np.int32)
    pos_b = np.stack([rng.choice(T, size=sb, replace=False) for _ in range(units)]).astype(np.int32)
    mask_a = (rng.random((units, sa)) < 0.6).astype(np.int32)
    n_a = np.array([sa, 50, 0, 96, 7], np.int32)
    n_b = np.array([sb, 40, 12, 0, 40], np.int32)
    dev = lambda x: torch.from_numpy(x).cuda()
    inter = torch.full((units,), -1, dtype=torch.int32, device="cuda")
    uni = torch.full((units,), -1, dtype=torch.int32, device="cuda")
    for use_mask in (True, False):
        roco.roco_set_overlap(dev(pos_a), dev(mask_a) if use_mask else None, dev(n_a), dev(pos_b), None, dev(n_b), T, inter, uni)
        torch.cuda.synchronize()
        for u in range(units):
            A = {int(p) for j, p in enumerate(pos_a[u, :n_a[u]]) if not use_mask or mask_a[u, j]}
            Bs = {int(p) for p in pos_b[u, :n_b[u]]}
            assert int(inter[u]) == len(A & Bs) and int(uni[u]) == len(A | Bs), (use_mask, u)


def test_set_overlap_over_the_largest_position_range():
    """max_pos = 524288, the documented limit: the bitmap alone fills 64 KiB of LDS, so the kernel's limit has to be
    raised; positions at both ends of the range, and one past it that must be ignored."""
    import paper_2402_06262_amd as roco
    T = 1 << 19
    rng = np.random.default_rng(11)
    units, sa, sb = 3, 512, 384
    pos_a = np.stack([rng.choice(T, size=sa, replace=False) for _ in range(units)]).astype(np.int32)
    pos_b = np.stack([rng.choice(T, size=sb, replace=False) for _ in range(units)]).astype(np.int32)
    pos_a[:, 0], pos_a[:, 1] = 0, T - 1
    pos_b[:, 0], pos_b[:, 1], pos_b[:, 2] = T - 1, 0, T  # the last one lies outside [0, max_pos)
    pos_b[:, 3:200] = pos_a[:, 3:200]  # a large common part
    n_a = np.full(units, sa, np.int32)
    n_b = np.array([sb, 100, 3], np.int32)
    dev = lambda x: torch.from_numpy(x).cuda()
    inter = torch.full((units,), -1, dtype=torch.int32, device="cuda")
    uni = torch.full((units,), -1, dtype=torch.int32, device="cuda")
    roco.roco_set_overlap(dev(pos_a), None, dev(n_a), dev(pos_b), None, dev(n_b), T, inter, uni)
    torch.cuda.synchronize()
    for u in range(units):
        A = {int(p) for p in pos_a[u, :n_a[u]]}
        Bs = {int(p) for p in pos_b[u, :n_b[u]] if p < T}
        assert int(inter[u]) == len(A & Bs) and int(uni[u]) == len(A | Bs), u
