"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

All units of a workload (or of one layer of it) run on the GPU; a seeded sample of units is compared with the
float64 oracle element by element (prefill statistics, retained sets, cached rows; then lock-step decode:
outputs, victims, statistics), and properties that hold at any size are checked on every unit:
Count = L - pos, ascending unique positions, cached rows equal the prompt rows they came from, one eviction per
full unit per step, softmax rows summing to one (the sum of the Acc increments of a step is 1 per unit).
"""
import math
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from inputs import CONFIGS, make_unit, unit_ids
from inputs.device import make_layer_on_device
from oracle import roco_oracle as orc

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1200)]


def _P():
    import parity
    return parity


def generate(cfg, ids, workers=None):
    T, d = cfg.total_len, cfg.head_dim
    Q = np.empty((len(ids), T, d), np.float32)
    K = np.empty_like(Q)
    V = np.empty_like(Q)

    def one(i):
        u = make_unit(cfg, *ids[i])
        Q[i], K[i], V[i] = u.Q, u.K, u.V

    with ThreadPoolExecutor(workers or min(16, len(os.sched_getaffinity(0)))) as ex:
        list(ex.map(one, range(len(ids))))
    return Q, K, V


def upload(x, dt, chunk=32):
    out = torch.empty(x.shape, dtype=dt, device="cuda")
    for i in range(0, x.shape[0], chunk):
        out[i:i + chunk] = torch.from_numpy(np.ascontiguousarray(x[i:i + chunk])).cuda().to(dt)
    return out


def run_case(cfg, ids, sample, decode_steps, scopes, tag, want_out=False, out_rows=None, shared=None):
    """`shared`: a dict that keeps the generated inputs, their device copies and the oracle's prompt statistics
    between calls (several tests on one workload)."""
    import paper_2402_06262_amd as roco
    P = _P()
    L, B, d = cfg.prompt_len, cfg.budget, cfg.head_dim
    U = len(ids)
    sc = 1.0 / math.sqrt(d)
    dt = P.torch_dtype(cfg.dtype)
    shared = {} if shared is None else shared
    if "Q" not in shared:
        print(f"[{tag}] generating {U} units, L={L}, B={B}, d={d}", flush=True)
        shared["Q"], shared["K"], shared["V"] = generate(cfg, ids)
        shared["dev"] = tuple(upload(shared[n][:, :L], dt) for n in "QKV")
        shared["full_stats"] = {}
    Q, K, V = shared["Q"], shared["K"], shared["V"]
    dQ, dK, dV = shared["dev"]
    dlen = torch.full((U,), L, dtype=torch.int32, device="cuda")
    total = P.TieCount()
    full_stats = shared["full_stats"]
    for scope in scopes:
        sess = P.make_session(U, d, B, scope, cfg.dtype, 0.0, cfg.recency_window, cfg.recency_bias)
        p, c = sess.params, sess.cache
        ws = torch.empty(roco.prefill_workspace_bytes(p, L), dtype=torch.uint8, device="cuda")
        O = torch.zeros_like(dQ) if want_out else None
        print(f"[{tag}] prefill_compress scope={scope}", flush=True)
        roco.roco_prefill_compress(p, dQ, dK, dV, dlen, L, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, O, ws)
        torch.cuda.synchronize()
        # ---- properties on every unit
        assert bool((c.n_used == min(L, B)).all())
        pos = c.pos.long()
        assert bool((pos[:, 1:] > pos[:, :-1]).all()) and int(pos.min()) >= 0 and int(pos.max()) < L
        assert bool((c.stats[:, 2] == (L - pos).float()).all()), "Count must equal L - pos on every unit"
        idx = pos[:, :, None].expand(U, B, d)
        assert torch.equal(torch.gather(dK, 1, idx), c.K) and torch.equal(torch.gather(dV, 1, idx), c.V)
        assert bool((c.stats[:, 0] > 0).all()) and bool((c.stats[:, 0] <= c.stats[:, 2]).all())
        assert bool((c.next_slot >= 0).all()) and bool((c.next_slot < B).all())
        # ---- sampled units against the oracle
        g = dict(K=None, V=None, stats=P.to_host(c.stats[sample]), pos=P.to_host(c.pos[sample]),
                 n_used=P.to_host(c.n_used[sample]), O=None if O is None else P.to_host(O[sample]))
        g["K"], g["V"] = P.to_host(c.K[sample]), P.to_host(c.V[sample])
        states = []
        for k, u in enumerate(sample):
            if u not in full_stats:
                print(f"[{tag}] oracle statistics of unit {u}", flush=True)
                full_stats[u] = orc.prefill_statistics(Q[u, :L], K[u, :L], V[u, :L], L, sc, cfg.recency_window,
                                                       cfg.recency_bias, want_out)
            res, t = P.check_prefill_unit(g, k, Q[u, :L], K[u, :L], V[u, :L], L, B, scope, sc, cfg.dtype,
                                          cfg.recency_window, cfg.recency_bias, want_out, full=full_stats[u],
                                          out_rows=out_rows)
            total += t
            states.append(res.cache)
        if decode_steps == 0:
            continue
        # ---- decode: every unit steps on the GPU, the sample is compared in lock-step
        sq, sk, sv = (upload(np.ascontiguousarray(x[:, L:L + decode_steps].transpose(1, 0, 2)), dt) for x in (Q, K, V))
        out = torch.empty((U, d), dtype=dt, device="cuda")
        ev_slot = torch.empty((U,), dtype=torch.int32, device="cuda")
        ev_pos = torch.empty_like(ev_slot)
        wsd = torch.empty(roco.decode_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        sidx = torch.tensor(sample, device="cuda")
        for step in range(decode_steps):
            t = L + step
            qpos = torch.full((U,), t, dtype=torch.int32, device="cuda")
            acc_before = c.stats[:, 0].double().sum(1)
            roco.roco_decode_step(p, sq[step], sk[step], sv[step], qpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot,
                                  out, ev_slot, ev_pos, wsd)
            if step % 16 == 0 or step == decode_steps - 1:  # any-size properties, on every unit
                assert bool((ev_slot >= 0).all()) and bool((ev_slot < B).all())
                assert bool((torch.gather(c.pos, 1, ev_slot.long()[:, None])[:, 0] == t).all())
                assert bool((c.n_used == B).all())
                assert bool(torch.isfinite(out.float()).all())
            g_out, g_slot, g_pos = P.to_host(out[sidx]), P.to_host(ev_slot[sidx]), P.to_host(ev_pos[sidx])
            for k, u in enumerate(sample):
                # rows sum to one: the step added p to every slot and reset the victim's Acc first
                victim_acc = states[k].acc[int(g_slot[k])]
                total += P.lockstep_decode_unit(states[k], k, g_out, g_slot, g_pos, Q[u, t], K[u, t], V[u, t], t,
                                                scope, sc, cfg.dtype, cfg.recency_window, cfg.recency_bias,
                                                what=f"[{tag}] scope {scope} step {step} unit {u}")
                if step % 16 == 0:
                    inc = float(c.stats[u, 0].double().sum() - acc_before[u]) + victim_acc
                    assert abs(inc - 1.0) < 2e-3, f"[{tag}] unit {u} step {step}: Acc increments sum to {inc}"
            if step % 64 == 63 or step == decode_steps - 1:
                host = dict(K=P.to_host(c.K[sidx]), V=P.to_host(c.V[sidx]), stats=P.to_host(c.stats[sidx]),
                            pos=P.to_host(c.pos[sidx]), n_used=P.to_host(c.n_used[sidx]))
                for k, u in enumerate(sample):
                    P.check_cache_unit(host, k, states[k], what=f"[{tag}] scope {scope} step {step} unit {u}")
        del sq, sk, sv
    print(f"[{tag}] declared ties: {total}", flush=True)
    P.assert_few_ties(total, tag)
    return total


def test_config2_prefill_4096_to_2048_scope_128():
    cfg = CONFIGS[1]
    ids = unit_ids(cfg)
    run_case(cfg, ids, sample=[0, 13, 31], decode_steps=0, scopes=[cfg.scope], tag="cfg2")


def test_config2_prefill_with_attention_output():
    """Same workload with the attention output O requested (matrix-core kernel with the P.V product)."""
    cfg = CONFIGS[1]
    ids = unit_ids(cfg)
    rows = [0, 1, 2, 31, 32, 33, 63, 64, 127, 128, 129, 1000, 2047, 2048, 3000, 4094, 4095]
    run_case(cfg, ids, sample=[0, 17], decode_steps=0, scopes=[cfg.scope], tag="cfg2-out", want_out=True, out_rows=rows)


def test_config3_serving_shape_prefill_and_lockstep_decode():
    """All 512 units (batch 16 x 32 heads), 3072 -> 2048, scope 64; all 512 decode steps in lock-step on 8 units."""
    cfg = CONFIGS[2]
    ids = unit_ids(cfg)
    sample = [0, 77, 130, 255, 300, 388, 470, 511]
    t = run_case(cfg, ids, sample=sample, decode_steps=cfg.steps, scopes=[cfg.scope], tag="cfg3")
    assert t.decode_decisions == len(sample) * cfg.steps


def test_config4_all_32_layers_as_one_batch_of_8192_units():
    """Workload 4 as stated: 32 layers x 8 sequences x 32 heads = 8192 units, 8192 -> 1024, scope 32, heavy-hitter
    fraction 0.5 % .. 5 % across the layers.  The prompt pass runs layer by layer (256 units per call, as a model
    would call it) into slices of ONE cache; every one of the 256 decode steps is a single 8192-unit
    roco_decode_step launch (16 rounds of workgroups on the chip).  Units sampled from the first, a middle and the
    last layer are compared with the oracle in lock-step; the any-size properties are checked on all 8192 units."""
    import paper_2402_06262_amd as roco
    P = _P()
    cfg = CONFIGS[3]
    L, B, d, steps, scope = cfg.prompt_len, cfg.budget, cfg.head_dim, cfg.steps, cfg.scope
    per_layer = cfg.batch * cfg.heads
    U = cfg.units
    assert U == 8192 and per_layer == 256
    sc = 1.0 / math.sqrt(d)
    dt = P.torch_dtype(cfg.dtype)
    sample = [5, 200, 15 * per_layer + 100, 31 * per_layer + 3, 31 * per_layer + 255]  # global unit ids
    sess = P.make_session(U, d, B, scope, cfg.dtype)
    c = sess.cache
    lp = roco.RocoParams(per_layer, d, B, scope, roco.ROCO_BF16)
    ws = torch.empty(roco.prefill_workspace_bytes(lp, L), dtype=torch.uint8, device="cuda")
    dlen = torch.full((per_layer,), L, dtype=torch.int32, device="cuda")
    sq = torch.empty((steps, U, d), dtype=dt, device="cuda")
    sk, sv = torch.empty_like(sq), torch.empty_like(sq)
    kept = {}  # sampled unit -> its host inputs
    total = P.TieCount()
    states = {}
    for layer in range(cfg.layers):
        # drawn on the device (the host generator would need minutes for 8192 units); sampled units are copied back
        Qd, Kd, Vd, _ = make_layer_on_device(cfg, layer)
        lo, hi = layer * per_layer, (layer + 1) * per_layer
        dQ, dK, dV = Qd[:, :L].contiguous(), Kd[:, :L].contiguous(), Vd[:, :L].contiguous()
        roco.roco_prefill_compress(lp, dQ, dK, dV, dlen, L, c.K[lo:hi], c.V[lo:hi], c.stats[lo:hi], c.pos[lo:hi],
                                   c.n_used[lo:hi], c.next_slot[lo:hi], None, ws)
        for x, dst in ((Qd, sq), (Kd, sk), (Vd, sv)):
            dst[:, lo:hi] = x[:, L:L + steps].transpose(0, 1)
        torch.cuda.synchronize()
        pos = c.pos[lo:hi].long()
        idx = pos[:, :, None].expand(per_layer, B, d)
        assert torch.equal(torch.gather(dK, 1, idx), c.K[lo:hi]) and torch.equal(torch.gather(dV, 1, idx), c.V[lo:hi])
        for u in sample:
            if lo <= u < hi:
                kept[u] = tuple(P.to_host(x[u - lo]) for x in (Qd, Kd, Vd))
        del dQ, dK, dV, Qd, Kd, Vd
    # ---- properties of the compressed caches, all 8192 units
    pos = c.pos.long()
    assert bool((c.n_used == B).all())
    assert bool((pos[:, 1:] > pos[:, :-1]).all()) and int(pos.min()) >= 0 and int(pos.max()) < L
    assert bool((c.stats[:, 2] == (L - pos).float()).all())
    assert bool((c.next_slot >= 0).all()) and bool((c.next_slot < B).all())
    sidx = torch.tensor(sample, device="cuda")
    g = dict(K=P.to_host(c.K[sidx]), V=P.to_host(c.V[sidx]), stats=P.to_host(c.stats[sidx]), pos=P.to_host(c.pos[sidx]),
             n_used=P.to_host(c.n_used[sidx]), O=None)
    for k, u in enumerate(sample):
        Qu, Ku, Vu = kept[u]
        print(f"[cfg4] oracle statistics of unit {u}", flush=True)
        res, t = P.check_prefill_unit(g, k, Qu[:L], Ku[:L], Vu[:L], L, B, scope, sc, cfg.dtype, want_out=False)
        total += t
        states[u] = res.cache
    # ---- 256 decode steps, each ONE launch over all 8192 units
    p = sess.params
    assert roco.decode_step_launches(p) == 1
    out = torch.empty((U, d), dtype=dt, device="cuda")
    ev_slot = torch.empty((U,), dtype=torch.int32, device="cuda")
    ev_pos = torch.empty_like(ev_slot)
    for step in range(steps):
        t = L + step
        qpos = torch.full((U,), t, dtype=torch.int32, device="cuda")
        check_all = step % 32 == 0 or step == steps - 1
        if check_all:
            acc_before = c.stats[:, 0].double().sum(1)
            victim_acc = None
        roco.roco_decode_step(p, sq[step], sk[step], sv[step], qpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, out,
                              ev_slot, ev_pos, sess.decode_ws)
        if check_all:  # on every unit
            assert bool((ev_slot >= 0).all()) and bool((ev_slot < B).all())
            assert bool((torch.gather(c.pos, 1, ev_slot.long()[:, None])[:, 0] == t).all())
            assert bool((c.n_used == B).all())
            assert bool(torch.isfinite(out.float()).all())
            # the three statistics of the slot just written: one observation by its own query
            fresh = torch.gather(c.stats, 2, ev_slot.long()[:, None, None].expand(U, 3, 1))[:, :, 0]
            assert bool((fresh[:, 2] == 1.0).all()) and bool((fresh[:, 0] > 0).all())
            assert bool(((fresh[:, 1] - fresh[:, 0] ** 2).abs() <= 1e-6 * fresh[:, 0] ** 2 + 1e-30).all())
        g_out, g_slot, g_pos = P.to_host(out[sidx]), P.to_host(ev_slot[sidx]), P.to_host(ev_pos[sidx])
        for k, u in enumerate(sample):
            Qu, Ku, Vu = kept[u]
            va = states[u].acc[int(g_slot[k])]
            total += P.lockstep_decode_unit(states[u], k, g_out, g_slot, g_pos, Qu[t], Ku[t], Vu[t], t, scope, sc,
                                            cfg.dtype, what=f"[cfg4] step {step} unit {u}")
            if check_all:  # softmax rows sum to one: the Acc increments of the step add up to 1
                inc = float(c.stats[u, 0].double().sum() - acc_before[u]) + va
                assert abs(inc - 1.0) < 2e-3, f"[cfg4] unit {u} step {step}: Acc increments sum to {inc}"
        if step % 64 == 63 or step == steps - 1:
            host = dict(K=P.to_host(c.K[sidx]), V=P.to_host(c.V[sidx]), stats=P.to_host(c.stats[sidx]),
                        pos=P.to_host(c.pos[sidx]), n_used=P.to_host(c.n_used[sidx]))
            for k, u in enumerate(sample):
                P.check_cache_unit(host, k, states[u], what=f"[cfg4] step {step} unit {u}")
    # every unit saw `steps` queries more: Count of a surviving prompt token is L - pos + steps
    pos = c.pos.long()
    assert bool((c.stats[:, 2] == (L + steps - pos).float()).all())
    print(f"[cfg4] declared ties: {total}", flush=True)
    assert total.decode_decisions == len(sample) * steps
    P.assert_few_ties(total, "cfg4")


_CFG5 = {}  # inputs and oracle prompt statistics of workload 5, shared by the four scopes


@pytest.mark.parametrize("scope", CONFIGS[4].scope_sweep)
def test_config5_long_context_all_1024_steps_for_each_scope(scope):
    """Workload 5 as stated: 40 heads, 32768 -> 4096 with the recency bias, then all 1024 decode steps at B = 4096;
    one test per scope of the sweep 16 / 64 / 256 / 1024 (the prompt and its oracle statistics are shared)."""
    cfg = CONFIGS[4]
    ids = unit_ids(cfg)
    t = run_case(cfg, ids, sample=[3, 21, 38], decode_steps=cfg.steps, scopes=[scope], tag=f"cfg5-s{scope}", shared=_CFG5)
    assert t.decode_decisions == 3 * cfg.steps
    if scope == cfg.scope_sweep[-1]:
        _CFG5.clear()


def test_hand_worked_six_token_example_through_the_library():
    """The 6-token example of tests/golden (exact rationals from the closed form P[i,j] = w_j / (w_0 + .. + w_i)),
    embedded in head_dim 64, fp32: q_i = e_0, k_j = ln(w_j) e_0, scale 1, v_j = (j + 1) e_0.  Prefill to budget 3 with
    scope 2 must retain positions {0, 1, 3}; the decode step (w = 3, v = 7) must evict slot 1 / position 1 and
    return 33/9; statistics as listed, at 1e-3."""
    import paper_2402_06262_amd as roco
    from fractions import Fraction as Fr
    P = _P()
    rec = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "six_token_example.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, *vals = line.split()
                rec[key] = [float(Fr(v)) for v in vals]
    w = rec["w"]
    L, B, s, d = 6, int(rec["budget"][0]), int(rec["scope"][0]), 64
    Q = np.zeros((1, L + 1, d), np.float32)
    K = np.zeros_like(Q)
    V = np.zeros_like(Q)
    Q[0, :, 0] = 1.0
    K[0, :L, 0] = np.log(np.array(w))
    K[0, L, 0] = math.log(rec["decode_w"][0])
    V[0, :L, 0] = np.arange(1, L + 1)
    V[0, L, 0] = 7.0
    for fused in ("0", "1"):
        os.environ["ROCO_DECODE_FUSED"] = fused
        try:
            sess = P.make_session(1, d, B, s, "f32", scale=1.0)
            g = P.gpu_prefill(sess, Q[:, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), [L], True)
            retained = [int(x) for x in rec["retained"]]
            assert g["pos"][0].tolist() == retained and int(g["n_used"][0]) == B
            for plane, name in ((0, "acc"), (1, "acc2"), (2, "count")):
                want = np.array([rec[name][j] for j in retained])
                assert np.allclose(g["stats"][0, plane], want, rtol=1e-3, atol=0), (name, g["stats"][0, plane], want)
            rows = [rec[f"row{i}"] for i in range(L)]
            for i in range(L):  # attention output of the prompt: sum_j P[i,j] (j + 1)
                assert abs(g["O"][0, i, 0] - sum(pj * (j + 1) for j, pj in enumerate(rows[i]))) < 1e-3 * 6
            out, ev_slot, ev_pos = P.gpu_decode_step(sess, Q[:, L], K[:, L], V[:, L], [L])
            assert int(ev_slot[0]) == int(rec["decode_evicted_slot"][0]) and int(ev_pos[0]) == int(rec["decode_evicted_pos"][0])
            assert abs(out[0, 0] - rec["decode_out"][0]) < 1e-3 * rec["decode_out"][0] and np.all(out[0, 1:] == 0.0)
            host = P.cache_to_host(sess)
            assert host["pos"][0].tolist() == [0, 6, 3]
            for plane, name in ((0, "decode_acc"), (1, "decode_acc2"), (2, "decode_count")):
                assert np.allclose(host["stats"][0, plane], rec[name], rtol=1e-3, atol=0), (name, host["stats"][0, plane])
        finally:
            os.environ.pop("ROCO_DECODE_FUSED", None)
