"""GPU parity of the block-wise evict-and-encode step (roco_encode_block) with the oracle."""
import math

import numpy as np
import pytest
import torch

from inputs import CONFIGS, make_unit, round_to_bf16
from oracle import roco_oracle as orc

pytestmark = pytest.mark.gpu


def _P():
    import parity
    return parity


def drive(units, d, B, s, prompt_lens, blocks, seed, recency=False, tag=""):
    """Optional prefill-compress of `prompt_lens`, then a sequence of block steps of the given sizes."""
    import paper_2402_06262_amd as roco
    P = _P()
    sc = 1.0 / math.sqrt(d)
    Lmax = max(max(prompt_lens), 1)
    T = Lmax + sum(blocks)
    rng = np.random.default_rng(seed)
    Q = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32) + 0.25)
    K = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    kw = dict(recency_window=24, recency_bias=0.5) if recency else {}
    sess = P.make_session(units, d, B, s, "bf16", 0.0, *(kw.values() if recency else ()))
    rw, rb = (24, 0.5) if recency else (0, 0.0)
    states, nxt = [], []
    if max(prompt_lens) > 0:
        g = P.gpu_prefill(sess, Q[:, :Lmax].copy(), K[:, :Lmax].copy(), V[:, :Lmax].copy(), prompt_lens, False)
        for u in range(units):
            res, _ = P.check_prefill_unit(g, u, Q[u, :Lmax], K[u, :Lmax], V[u, :Lmax], prompt_lens[u], B, s, sc, "bf16",
                                          rw, rb, False)
            states.append(res.cache)
            nxt.append(prompt_lens[u])
    else:
        for u in range(units):
            states.append(orc.CacheState(np.zeros((B, d)), np.zeros((B, d)), np.zeros(B), np.zeros(B), np.zeros(B),
                                         np.full(B, -1, dtype=np.int64), 0))
            nxt.append(0)
    ties = P.TieCount()
    t = Lmax
    for b in blocks:
        ws = torch.empty(max(16, roco.block_workspace_bytes(sess.params, b)), dtype=torch.uint8, device="cuda")
        print(f"[{tag}] block of {b} at row {t}", flush=True)
        g_out, g_slot, g_pos = P.gpu_encode_block(sess, b, Q[:, t:t + b], K[:, t:t + b], V[:, t:t + b], nxt, ws)
        for u in range(units):
            ties += P.lockstep_block_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t:t + b], K[u, t:t + b], V[u, t:t + b],
                                          nxt[u], s, sc, "bf16", rw, rb, what=f"[{tag}] block {b} @ {t}")
            assert states[u].n_used <= B
        host = P.cache_to_host(sess)
        for u in range(units):
            P.check_cache_unit(host, u, states[u], what=f"[{tag}] after block {b} @ {t}")
        nxt = [p + b for p in nxt]
        t += b
    # the hint left for a following single-token step is the oracle's victim on the final statistics
    g_out, g_slot, g_pos = P.gpu_decode_step(sess, Q[:, t - 1], K[:, t - 1], V[:, t - 1], nxt)
    for u in range(units):
        ties += P.lockstep_decode_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t - 1], K[u, t - 1], V[u, t - 1], nxt[u], s,
                                       sc, "bf16", rw, rb, what=f"[{tag}] decode after blocks")
    print(f"[{tag}] ties {ties}", flush=True)
    return ties


@pytest.mark.parametrize("b", [1, 2, 5, 16, 32])
def test_block_steps_on_a_full_cache(b):
    """Cache filled by prefill-compress, then blocks of b tokens: b evictions per step."""
    drive(3, 128, 256, 24, [400, 300, 256], [b] * 4, seed=60 + b, tag=f"full-{b}")


def test_block_steps_fill_an_empty_cache_then_start_evicting():
    """Block-wise prompt encoding from scratch: no eviction until the budget is reached, partial eviction when a
    block straddles it, ragged block sizes."""
    drive(2, 128, 200, 16, [0, 0], [32, 32, 32, 32, 32, 32, 7, 32, 1, 13, 32], seed=71, tag="from-empty")


def test_block_steps_with_recency_bias_and_partially_filled_units():
    drive(3, 128, 128, 10, [100, 128, 60], [16, 16, 9, 32], seed=72, recency=True, tag="recency")


def test_block_step_many_splits_budget_2048():
    drive(2, 128, 2048, 64, [2300, 2048], [32, 16, 32], seed=73, tag="b2048")
