"""Tie-band check for eviction decisions.  TEST INFRASTRUCTURE ONLY.

The HIP path keeps Acc, Acc2 and Count in fp32 and the oracle keeps them in
float64, so the two may order two tokens differently when the oracle's own gap
between them is below what fp32 statistics can resolve.  The matching rule is:
index sets must be identical unless the oracle's own score gap lies inside the
tolerance band

    MAS:       |gap| <= rel * MAS
    variance:  |gap| <= rel * (Acc2/Count + MAS^2)          rel = 1e-5

(the variance band is stated on the two terms that cancel in
Acc2/Count - MAS^2, section 4.3 of the paper, because the difference itself can
be arbitrarily smaller than either).

`admissible_eviction` answers, for an eviction set G that differs from the
oracle's: is there an assignment of the in-band tokens to the two sides of the
variance threshold, and an ordering of in-band MAS values, under which RoCo's
rule evicts exactly G?  If so the case is a *declared tie*; the harness counts
it and lets the oracle adopt G so later steps stay comparable.  If not, the HIP
path is wrong.
"""
from __future__ import annotations

from typing import Iterable, Tuple

import numpy as np

F64 = np.float64

# Relative width of the band.  The statistics are fp32 sums of up to a few tens of thousands of probabilities, each
# itself good to a few ulp: rounding error accumulates like sqrt(N) * 2^-24, about 1e-5 for N = 32768.  (Every
# differing decision of the GPU suite lies inside 1e-6; at 1e-7, two ulp, some of them no longer do.)
REL = 1e-5


def bands_for(policy, acc, acc2, count, rel: float = REL) -> Tuple[np.ndarray, np.ndarray]:
    """(eps_importance, eps_scope_key) per token for an eviction policy (an object with `importance` and
    `scope_kind` strings, or None for RoCo): scores that are sums of probabilities get the relative band,
    scores that are positions are exact."""
    eps_m, eps_v = bands(acc, acc2, count, rel)
    importance = getattr(policy, "importance", "mas")
    scope_kind = getattr(policy, "scope_kind", "std")
    if importance == "aas":
        eps_m = rel * np.abs(np.asarray(acc, dtype=F64))
    elif importance == "ltas":
        eps_m = rel * np.abs(np.asarray(acc2, dtype=F64))  # the second array holds the score itself
    elif importance == "oldest":
        eps_m = np.zeros_like(eps_m)
    if scope_kind != "std":
        eps_v = np.zeros_like(eps_v)
    return eps_m, eps_v


def bands(acc, acc2, count, rel: float = REL) -> Tuple[np.ndarray, np.ndarray]:
    """(eps_mas, eps_var) per token."""
    acc, acc2, count = (np.asarray(a, dtype=F64) for a in (acc, acc2, count))
    mas = acc / count
    return rel * np.abs(mas), rel * (acc2 / count + mas * mas)


def admissible_eviction(mas, var, eps_mas, eps_var, scope: int, n_evict: int,
                        evicted: Iterable[int]) -> Tuple[bool, str]:
    """Can RoCo's rule, with in-band comparisons decided either way, evict exactly `evicted`?"""
    mas, var = np.asarray(mas, dtype=F64), np.asarray(var, dtype=F64)
    n = mas.shape[0]
    G = np.array(sorted(int(g) for g in evicted), dtype=np.int64)
    if G.shape[0] != n_evict or np.unique(G).shape[0] != n_evict:
        return False, "wrong number of evicted tokens"
    if n_evict == 0:
        return True, "nothing to evict"
    if G.min() < 0 or G.max() >= n:
        return False, "evicted index out of range"
    m = min(n, scope + n_evict - 1)
    order = np.argsort(var, kind="stable")
    t = order[m - 1]
    if m == n:
        border = np.zeros(n, dtype=bool)
        inside = np.ones(n, dtype=bool)
    else:
        border = np.abs(var - var[t]) <= eps_var + eps_var[t]
        inside = (var < var[t]) & ~border  # in the scope whatever the in-band order is
    outside = ~inside & ~border
    in_G = np.zeros(n, dtype=bool)
    in_G[G] = True
    if np.any(outside & in_G):
        return False, "an evicted token lies clearly outside the variance scope"
    # every scope member that survives must not have a clearly lower MAS than an evicted one
    thr = np.max(mas[G] - eps_mas[G])
    survives_ok = mas + eps_mas >= thr
    if np.any(inside & ~in_G & ~survives_ok):
        return False, "a token clearly inside the scope with clearly lower MAS was kept"
    fixed = int(np.count_nonzero(inside | (border & in_G)))
    if fixed > m:
        return False, "more in-band tokens evicted than the scope can hold"
    fill = int(np.count_nonzero(border & ~in_G & survives_ok))
    if fixed + fill < m:
        return False, "scope cannot be completed without a token of clearly lower MAS"
    return True, "declared tie"
