"""Consistency study of section 4.1 (Fig. 2) on synthetic data, driven entirely through the HIP library.

For an importance score, a cache budget B and every sampled position t of a sequence, two sets of B tokens are
compared by Jaccard similarity: the tokens a budgeted cache holds after step t (it only ever saw the attention
its own B slots received), and the B most important tokens when the full cache is available (statistics of all
t + 1 tokens, from a run that never evicts).  The paper sets the local window to 0, i.e. the scope is the whole
cache, and averages over positions, heads and layers; here the average runs over positions and units.

Everything the method computes (attention, statistics, evictions, the top-B selection, the overlap of the two sets)
runs in the library's kernels; this module only steps the two caches side by side and averages the ratios.
"""
from __future__ import annotations

from typing import Optional, Dict, Iterable, Sequence, Tuple

from . import binding as roco

IMPORTANCE = {"mas": roco.ROCO_IMPORTANCE_MAS, "aas": roco.ROCO_IMPORTANCE_AAS, "oldest": roco.ROCO_IMPORTANCE_OLDEST,
              "ltas": roco.ROCO_IMPORTANCE_LAST, "aqas": roco.ROCO_IMPORTANCE_COUNT}
# what the second statistics plane holds under each importance: scores that share it can share a full-cache run
_SECOND = {"ltas": "last", "aqas": "count"}


class _Run:
    """One cache stepped token by token."""

    def __init__(self, torch, params, L_max):
        self.torch, self.p = torch, params
        self.cache = roco.alloc_cache(params)
        self.ws_d = torch.empty(max(16, roco.decode_workspace_bytes(params)), dtype=torch.uint8, device="cuda")
        self.ws_p = torch.empty(max(16, roco.prefill_workspace_bytes(params, L_max)), dtype=torch.uint8, device="cuda")
        self.out = torch.empty((params.units, params.head_dim), dtype=torch.bfloat16 if params.dtype == roco.ROCO_BF16
                               else torch.float32, device="cuda")

    def prefill(self, Q, K, V, lens, L):
        c = self.cache
        roco.roco_prefill_compress(self.p, Q, K, V, lens, L, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, None,
                                   self.ws_p)

    def step(self, q, k, v, qpos):
        c = self.cache
        roco.roco_decode_step(self.p, q, k, v, qpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, self.out, None,
                              None, self.ws_d)


def consistency_study(Q, K, V, prompt_len: int, rates: Sequence[float] = (0.3, 0.4, 0.5, 0.6),
                      importances: Iterable[str] = ("mas", "aas"), sample_every: int = 8,
                      sinks: int = 0, counts: Optional[dict] = None) -> Dict[str, Dict[float, Tuple[float, int]]]:
    """Q, K, V: device tensors [units, T, d] (bf16 or fp32), the first `prompt_len` rows are the prompt.

    Budget for rate r is round(r * T).  Returns {importance: {rate: (mean Jaccard, positions compared)}} over the
    sampled positions t >= prompt_len at which the full cache holds more than B tokens.  A dict passed as `counts`
    receives the raw set sizes behind every ratio: counts[(importance, rate, t)] = (|A and B|, |A or B|) per unit.
    """
    import torch
    U, T, d = Q.shape
    L = int(prompt_len)
    dt = roco.ROCO_BF16 if Q.dtype == torch.bfloat16 else roco.ROCO_F32
    lens = torch.full((U,), L, dtype=torch.int32, device="cuda")
    Qp, Kp, Vp = (x[:, :L].contiguous() for x in (Q, K, V))
    steps = [(Q[:, t].contiguous(), K[:, t].contiguous(), V[:, t].contiguous(),
              torch.full((U,), t, dtype=torch.int32, device="cuda")) for t in range(L, T)]
    sampled = [t for t in range(L, T) if (t - L) % sample_every == sample_every - 1 or t == T - 1]

    # the full-cache runs: the statistics do not depend on the policy (one run serves every importance and rate),
    # except for what the second plane holds (squares, the latest query's attention, or the thresholded count)
    importances = list(importances)
    fulls = {}
    for second in sorted({_SECOND.get(name, "square") for name in importances}):
        imp = {"square": roco.ROCO_IMPORTANCE_MAS, "last": roco.ROCO_IMPORTANCE_LAST,
               "count": roco.ROCO_IMPORTANCE_COUNT}[second]
        fulls[second] = _Run(torch, roco.RocoParams(U, d, T, T, dt, importance=imp, scope_kind=roco.ROCO_SCOPE_ALL), L)
        fulls[second].prefill(Qp, Kp, Vp, lens, L)
    budgets = {r: max(1, min(T, int(round(r * T)))) for r in rates}
    runs = {}
    for name in importances:
        for r, B in budgets.items():
            p = roco.RocoParams(U, d, B, B, dt, importance=IMPORTANCE[name], scope_kind=roco.ROCO_SCOPE_ALL, sinks=sinks)
            run = _Run(torch, p, L)
            run.prefill(Qp, Kp, Vp, lens, L)
            runs[(name, r)] = run
    total = {key: 0.0 for key in runs}
    count = {key: 0 for key in runs}
    mask = torch.empty((U, T), dtype=torch.int32, device="cuda")
    inter = torch.empty((U,), dtype=torch.int32, device="cuda")
    union = torch.empty((U,), dtype=torch.int32, device="cuda")
    for i, t in enumerate(range(L, T)):
        q, k, v, qpos = steps[i]
        for full in fulls.values():
            full.step(q, k, v, qpos)
        for run in runs.values():
            run.step(q, k, v, qpos)
        if t not in sampled:
            continue
        for (name, r), run in runs.items():
            full = fulls[_SECOND.get(name, "square")]
            fc = full.cache
            B = budgets[r]
            if t + 1 <= B:
                continue  # nothing has been evicted yet: the two sets are trivially equal
            sel = roco.RocoParams(U, d, T, T, dt, importance=IMPORTANCE[name], scope_kind=roco.ROCO_SCOPE_ALL, sinks=sinks)
            roco.roco_select_retained(sel, B, fc.stats, fc.pos, fc.n_used, mask, full.ws_d)
            c = run.cache
            roco.roco_set_overlap(fc.pos, mask, fc.n_used, c.pos, None, c.n_used, T, inter, union)
            i_h, u_h = inter.cpu().numpy(), union.cpu().numpy()  # the report: mean ratio over units and positions
            if counts is not None:
                counts[(name, r, t)] = (i_h.copy(), u_h.copy())
            total[(name, r)] += float((i_h / u_h).sum())
            count[(name, r)] += U
    torch.cuda.synchronize()
    out: Dict[str, Dict[float, Tuple[float, int]]] = {}
    for (name, r), s in total.items():
        out.setdefault(name, {})[r] = (s / count[(name, r)] if count[(name, r)] else float("nan"), count[(name, r)])
    return out
