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


def run_case(cfg, ids, sample, decode_steps, scopes, tag, want_out=False, out_rows=None):
    import paper_2402_06262_amd as roco
    P = _P()
    L, B, d = cfg.prompt_len, cfg.budget, cfg.head_dim
    U = len(ids)
    sc = 1.0 / math.sqrt(d)
    dt = P.torch_dtype(cfg.dtype)
    print(f"[{tag}] generating {U} units, L={L}, B={B}, d={d}", flush=True)
    Q, K, V = generate(cfg, ids)
    dQ, dK, dV = upload(Q[:, :L], dt), upload(K[:, :L], dt), upload(V[:, :L], dt)
    dlen = torch.full((U,), L, dtype=torch.int32, device="cuda")
    total = P.TieCount()
    full_stats = {}
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


def test_config4_two_layers_8192_to_1024():
    """Layers 0, 15 and 31 (heavy-hitter fraction 0.5 % .. 5 %), all 8 sequences x 32 heads each; all 256 decode steps."""
    cfg = CONFIGS[3]
    for layer in (0, 15, cfg.layers - 1):
        ids = [(layer, b, h) for b in range(cfg.batch) for h in range(cfg.heads)]
        run_case(cfg, ids, sample=[5, 100, 200], decode_steps=cfg.steps, scopes=[cfg.scope], tag=f"cfg4-layer{layer}")


def test_config5_long_context_scope_sweep_with_recency_bias():
    """40 heads, 32768 -> 4096 with the recency bias; scope sweep 16 / 64 / 256 / 1024; 128 decode steps each."""
    cfg = CONFIGS[4]
    ids = unit_ids(cfg)
    run_case(cfg, ids, sample=[3, 21, 38], decode_steps=128, scopes=list(cfg.scope_sweep), tag="cfg5")
