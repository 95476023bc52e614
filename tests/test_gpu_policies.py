"""GPU parity of the other eviction policies of the two-stage framework (importance x scope) with the oracle:
prefill-compress, token-wise decode on both shapes of the step, block-wise steps and the selection entry point."""
import math

import numpy as np
import pytest
import torch

from inputs import round_to_bf16
from oracle import roco_oracle as orc

pytestmark = pytest.mark.gpu

POLICIES = {
    "h2o": orc.Policy("aas", "window"),            # accumulated score, recent half protected
    "aas-all": orc.Policy("aas", "all"),
    "mas-window": orc.Policy("mas", "window"),     # the paper's scope study: mean score with a local window
    "aas-std": orc.Policy("aas", "std"),
    "sinks": orc.Policy("oldest", "all", 4),       # sliding window with four attention sinks
    "oldest-window": orc.Policy("oldest", "window", 2),
    "tova": orc.Policy("ltas", "all"),             # last-token attention score over the whole cache
    "ltas-window": orc.Policy("ltas", "window"),
    "scissorhands": orc.Policy("aqas", "window"),  # thresholded count, recent half protected
    "aqas-all": orc.Policy("aqas", "all"),
}


def _P():
    import parity
    return parity


@pytest.fixture(params=["split", "fused"])
def decode_path(request, monkeypatch):
    monkeypatch.setenv("ROCO_DECODE_FUSED", "1" if request.param == "fused" else "0")
    return request.param


@pytest.mark.parametrize("name", list(POLICIES))
@pytest.mark.parametrize("dtype,head_dim", [("bf16", 128), ("f32", 64)])
def test_prefill_and_decode_under_each_policy(name, dtype, head_dim, decode_path):
    import test_gpu_parity as T
    pol = POLICIES[name]
    budget = 96
    scope = budget // 2 if pol.scope_kind == "window" else 12
    T.run_workload(dtype, head_dim, 4, [230, 200, 96, 40], 230, budget, scope, 40, seed=300 + len(name),
                   want_out=False, tag=f"policy-{name}-{dtype}-{decode_path}", policy=pol)


def test_sink_policy_keeps_the_sinks_and_the_most_recent_tokens():
    """Closed form on the device state itself: after prefill and 50 steps the cache of every full unit holds
    positions 0..3 and the most recent B - 4."""
    import paper_2402_06262_amd as roco
    P = _P()
    pol = POLICIES["sinks"]
    U, d, B, L, steps = 3, 128, 64, 150, 50
    rng = np.random.default_rng(7)
    Q, K, V = (round_to_bf16(rng.standard_normal((U, L + steps, d)).astype(np.float32)) for _ in range(3))
    sess = P.make_session(U, d, B, 1, "bf16", policy=pol)
    P.gpu_prefill(sess, Q[:, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), [L] * U, False)
    for t in range(L, L + steps):
        _, slot, pos = P.gpu_decode_step(sess, Q[:, t], K[:, t], V[:, t], [t] * U)
        assert np.all(pos == t - (B - 4))
    host = P.cache_to_host(sess)
    want = list(range(4)) + list(range(L + steps - (B - 4), L + steps))
    for u in range(U):
        assert sorted(host["pos"][u].tolist()) == want


@pytest.mark.parametrize("name", ["h2o", "sinks", "mas-window", "tova", "scissorhands"])
def test_block_steps_under_each_policy(name):
    import test_gpu_block as TB
    pol = POLICIES[name]
    P = _P()
    units, d, B = 3, 128, 128
    s = B // 2 if pol.scope_kind == "window" else 16
    sc = 1.0 / math.sqrt(d)
    import paper_2402_06262_amd as roco
    rng = np.random.default_rng(400 + len(name))
    blocks = [8, 1, 1, 8, 32, 5, 1, 16]  # single-token blocks take a path of their own: book-keeping in the finish
    L = 200
    T = L + sum(blocks)
    Q = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32) + 0.25)
    K = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    sess = P.make_session(units, d, B, s, "bf16", policy=pol)
    lens = [L, 160, B]
    g = P.gpu_prefill(sess, Q[:, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), lens, False)
    states, nxt = [], list(lens)
    for u in range(units):
        res, _ = P.check_prefill_unit(g, u, Q[u, :L], K[u, :L], V[u, :L], lens[u], B, s, sc, "bf16", 0, 0.0, False,
                                      policy=pol)
        states.append(res.cache)
    t = L
    for b in blocks:
        ws = torch.empty(roco.block_workspace_bytes(sess.params, b), dtype=torch.uint8, device="cuda")
        g_out, g_slot, g_pos = P.gpu_encode_block(sess, b, Q[:, t:t + b], K[:, t:t + b], V[:, t:t + b], nxt, ws)
        for u in range(units):
            P.lockstep_block_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t:t + b], K[u, t:t + b], V[u, t:t + b],
                                  nxt[u], s, sc, "bf16", what=f"[{name}] block {b} @ {t}", policy=pol)
        host = P.cache_to_host(sess)
        for u in range(units):
            P.check_cache_unit(host, u, states[u], what=f"[{name}] after block {b}")
        nxt = [p + b for p in nxt]
        t += b
    # the victim kept for a following token-wise step is the policy's, and roco_select_victims reproduces it
    fresh = torch.full_like(sess.cache.next_slot, -9)
    c = sess.cache
    roco.roco_select_victims(sess.params, c.stats, c.pos, c.n_used, fresh, sess.decode_ws)
    torch.cuda.synchronize()
    assert torch.equal(fresh, c.next_slot)
    g_out, g_slot, g_pos = P.gpu_decode_step(sess, Q[:, t - 1], K[:, t - 1], V[:, t - 1], nxt)
    for u in range(units):
        P.lockstep_decode_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t - 1], K[u, t - 1], V[u, t - 1], nxt[u], s, sc,
                               "bf16", what=f"[{name}] decode after blocks", policy=pol)
