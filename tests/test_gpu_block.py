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


def drive(units, d, B, s, prompt_lens, blocks, seed, recency=False, tag="", dtype="bf16"):
    """Optional prefill-compress of `prompt_lens`, then a sequence of block steps of the given sizes."""
    import paper_2402_06262_amd as roco
    P = _P()
    sc = 1.0 / math.sqrt(d)
    Lmax = max(max(prompt_lens), 1)
    T = Lmax + sum(blocks)
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((units, T, d)).astype(np.float32) + 0.25
    K = rng.standard_normal((units, T, d)).astype(np.float32)
    V = rng.standard_normal((units, T, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    kw = dict(recency_window=24, recency_bias=0.5) if recency else {}
    sess = P.make_session(units, d, B, s, dtype, 0.0, *(kw.values() if recency else ()))
    rw, rb = (24, 0.5) if recency else (0, 0.0)
    states, nxt = [], []
    if max(prompt_lens) > 0:
        g = P.gpu_prefill(sess, Q[:, :Lmax].copy(), K[:, :Lmax].copy(), V[:, :Lmax].copy(), prompt_lens, False)
        for u in range(units):
            res, _ = P.check_prefill_unit(g, u, Q[u, :Lmax], K[u, :Lmax], V[u, :Lmax], prompt_lens[u], B, s, sc, dtype,
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
                                          nxt[u], s, sc, dtype, rw, rb, what=f"[{tag}] block {b} @ {t}")
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
                                       sc, dtype, rw, rb, what=f"[{tag}] decode after blocks")
    print(f"[{tag}] ties {ties}", flush=True)
    P.assert_few_ties(ties, tag)
    return ties


@pytest.mark.parametrize("b", [1, 2, 5, 16, 32, 33, 64])
def test_block_steps_on_a_full_cache(b):
    """Cache filled by prefill-compress, then blocks of b tokens: b evictions per step."""
    drive(3, 128, 256, 24, [400, 300, 256], [b] * 4, seed=60 + b, tag=f"full-{b}")


def test_single_token_blocks_with_the_preparing_kernel(monkeypatch):
    """Blocks of one token normally skip the preparing kernel; the general path must give the same step."""
    monkeypatch.setenv("ROCO_BLOCK_SINGLE", "0")
    drive(3, 128, 256, 24, [400, 300, 200], [1] * 70, seed=66, tag="prepared-1")


def test_single_token_blocks_fill_then_evict_with_recency_bias():
    drive(3, 128, 192, 16, [150, 192, 100], [1] * 100, seed=67, recency=True, tag="single-recency")


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 64), ("f32", 128)])
def test_block_steps_on_the_vector_path_for_other_dtypes_and_head_dims(dtype, d, monkeypatch):
    """Shapes the matrix-core kernel is not built for take the vector-ALU kernel (K and V streamed once for all query
    rows; its 8 / 16 / 32 / 64-row instantiations all run here): same step, same parity bar.  From a compressed cache
    and with a unit that is still filling up; ragged block sizes."""
    drive(3, d, 96, 10, [150, 96, 40], [8, 1, 32, 5, 16, 32, 3, 64, 47], seed=140 + d, tag=f"simple-{dtype}-{d}", dtype=dtype)
    drive(2, d, 64, 8, [100, 64], [4, 32], seed=150 + d, recency=True, tag=f"simple-recency-{dtype}-{d}", dtype=dtype)
    # eight splits of 128 slots over a budget that is no multiple of the 64-slot tile; a unit that stays far from full
    # ... with the non-temporal loads that caches larger than the last-level cache get
    monkeypatch.setenv("ROCO_STREAMING_LOADS", "1")
    drive(2, d, 1000, 24, [1100, 30], [64, 7, 16, 33, 2], seed=160 + d, tag=f"simple-splits-{dtype}-{d}", dtype=dtype)


def test_block_steps_fill_an_empty_cache_then_start_evicting():
    """Block-wise prompt encoding from scratch: no eviction until the budget is reached, partial eviction when a
    block straddles it, ragged block sizes."""
    drive(2, 128, 200, 16, [0, 0], [32, 32, 32, 32, 32, 32, 7, 32, 1, 13, 32], seed=71, tag="from-empty")
    drive(2, 128, 200, 16, [0, 0], [64, 64, 64, 64, 40, 64, 1, 64], seed=77, tag="from-empty-64")


def test_block_steps_with_recency_bias_and_partially_filled_units():
    drive(3, 128, 128, 10, [100, 128, 60], [16, 16, 9, 32], seed=72, recency=True, tag="recency")


def test_block_step_many_splits_budget_2048():
    drive(2, 128, 2048, 64, [2300, 2048], [32, 16, 32], seed=73, tag="b2048")


def test_block_steps_with_a_budget_above_4096():
    drive(1, 128, 4104, 40, [4200], [1, 1, 8, 32, 1, 3], seed=74, tag="b4104")


def test_block_steps_whose_ranking_keys_need_more_than_64_kib_of_lds():
    """8192 < B <= 16384: the preparing and finishing kernels raise their dynamic LDS limit before the launch."""
    drive(1, 128, 8200, 40, [8300], [1, 8, 32, 1], seed=75, tag="b8200")


def test_block_steps_with_a_budget_above_the_lds_key_limit():
    """B > 16384: the ranking keys of the preparing and finishing kernels live in the workspace."""
    drive(1, 128, 16392, 40, [16500], [1, 8, 32, 1], seed=76, tag="b16392")


def test_block_steps_at_the_serving_shape_all_512_units():
    """Workload 3's shape: all 512 units prefilled 3072 -> 2048, then blocks of 16 tokens; sampled units in
    lock-step with the oracle, any-size properties on every unit."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    import paper_2402_06262_amd as roco
    from inputs import unit_ids
    P = _P()
    cfg = CONFIGS[2]
    L, B, s, d, U = cfg.prompt_len, cfg.budget, cfg.scope, cfg.head_dim, cfg.units
    b, n_blocks = 16, 6
    ids = unit_ids(cfg)
    T = L + b * n_blocks
    Q = np.empty((U, T, d), np.float32); K = np.empty_like(Q); V = np.empty_like(Q)

    def one(i):
        un = make_unit(cfg, *ids[i], total_len=T)
        Q[i], K[i], V[i] = un.Q, un.K, un.V

    with ThreadPoolExecutor(min(16, len(os.sched_getaffinity(0)))) as ex:
        list(ex.map(one, range(U)))
    sc = 1.0 / math.sqrt(d)
    dtype = "bf16"
    sess = P.make_session(U, d, B, s, dtype)
    c, p = sess.cache, sess.params
    dt = torch.bfloat16
    up = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda().to(dt)
    dQ, dK, dV = up(Q[:, :L]), up(K[:, :L]), up(V[:, :L])
    dlen = torch.full((U,), L, dtype=torch.int32, device="cuda")
    wsp = torch.empty(roco.prefill_workspace_bytes(p, L), dtype=torch.uint8, device="cuda")
    roco.roco_prefill_compress(p, dQ, dK, dV, dlen, L, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, None, wsp)
    torch.cuda.synchronize()
    sample = [0, 101, 333, 511]
    states = [orc.prefill_compress(Q[u, :L], K[u, :L], V[u, :L], L, B, s, sc).cache for u in sample]
    for k, u in enumerate(sample):
        assert np.array_equal(c.pos[u].cpu().numpy(), states[k].pos)
    wsb = torch.empty(roco.block_workspace_bytes(p, b), dtype=torch.uint8, device="cuda")
    out = torch.empty((U, b, d), dtype=dt, device="cuda")
    es = torch.empty((U, b), dtype=torch.int32, device="cuda"); ep = torch.empty_like(es)
    sidx = torch.tensor(sample, device="cuda")
    ties = P.TieCount()
    for i in range(n_blocks):
        t = L + i * b
        qp0 = torch.full((U,), t, dtype=torch.int32, device="cuda")
        count_before = c.stats[:, 2].double().sum(1)
        roco.roco_encode_block(p, b, up(Q[:, t:t + b]), up(K[:, t:t + b]), up(V[:, t:t + b]), qp0, c.K, c.V, c.stats,
                               c.pos, c.n_used, c.next_slot, out, es, ep, wsb)
        torch.cuda.synchronize()
        assert bool((c.n_used == B).all()) and bool((es >= 0).all()) and bool((es < B).all())
        assert bool((torch.gather(c.pos, 1, es.long()) == (qp0[:, None] + torch.arange(b, device="cuda")[None])).all())
        assert bool(torch.isfinite(out.float()).all())
        assert bool((es[:, 1:] > es[:, :-1]).all())  # tokens take the freed slots in ascending order
        g_out, g_slot, g_pos = P.to_host(out[sidx]), P.to_host(es[sidx]), P.to_host(ep[sidx])
        for k, u in enumerate(sample):
            ties += P.lockstep_block_unit(states[k], k, g_out, g_slot, g_pos, Q[u, t:t + b], K[u, t:t + b], V[u, t:t + b],
                                          t, s, sc, dtype, what=f"[cfg3-block] block {i} unit {u}")
        host = dict(K=P.to_host(c.K[sidx]), V=P.to_host(c.V[sidx]), stats=P.to_host(c.stats[sidx]),
                    pos=P.to_host(c.pos[sidx]), n_used=P.to_host(c.n_used[sidx]))
        for k, u in enumerate(sample):
            P.check_cache_unit(host, k, states[k], what=f"[cfg3-block] block {i} unit {u}")
    print("[cfg3-block] ties", ties, flush=True)
    P.assert_few_ties(ties, "cfg3-block")


def test_block_steps_of_fp32_head_dim_64_at_the_benchmark_shape():
    """The shape bench.py times for the vector-ALU block kernel: 512 units x 2048 slots of fp32 / head_dim 64 (the
    non-temporal loads of a cache above the last-level cache's size, one split per unit).  Blocks of 64 fill the
    empty caches, then blocks of 64 / 16 / 8 / 1 / 33 evict (every instantiation of the kernel); sampled units in
    lock-step with the oracle, any-size properties on every unit."""
    import paper_2402_06262_amd as roco
    P = _P()
    U, d, B, s, dtype = 512, 64, 2048, 64, "f32"
    blocks = [64] * 32 + [64, 16, 8, 1, 33]
    T = sum(blocks)
    sc = 1.0 / math.sqrt(d)
    sess = P.make_session(U, d, B, s, dtype)
    c, p = sess.cache, sess.params
    gen = torch.Generator(device="cuda").manual_seed(4242)
    Q = torch.randn((U, T, d), device="cuda", generator=gen) + 0.25
    K = torch.randn((U, T, d), device="cuda", generator=gen)
    V = torch.randn((U, T, d), device="cuda", generator=gen)
    sample = [0, 201, 511]
    sidx = torch.tensor(sample, device="cuda")
    hQ, hK, hV = (P.to_host(x[sidx]).astype(np.float64) for x in (Q, K, V))
    states = [orc.CacheState(np.zeros((B, d)), np.zeros((B, d)), np.zeros(B), np.zeros(B), np.zeros(B),
                             np.full(B, -1, dtype=np.int64), 0) for _ in sample]
    ws = torch.empty(roco.block_workspace_bytes(p, 64), dtype=torch.uint8, device="cuda")
    ties = P.TieCount()
    t = 0
    for i, b in enumerate(blocks):
        print(f"[f32-d64-block] block {i} of {b} at row {t}", flush=True)
        out = torch.empty((U, b, d), dtype=torch.float32, device="cuda")
        es = torch.empty((U, b), dtype=torch.int32, device="cuda"); ep = torch.empty_like(es)
        qp0 = torch.full((U,), t, dtype=torch.int32, device="cuda")
        roco.roco_encode_block(p, b, Q[:, t:t + b].contiguous(), K[:, t:t + b].contiguous(), V[:, t:t + b].contiguous(), qp0,
                               c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, out, es, ep, ws)
        torch.cuda.synchronize()
        n_after = min(B, t + b)
        assert bool((c.n_used == n_after).all()) and bool(torch.isfinite(out).all())
        if t >= B:  # every token of the block took over an evicted token's slot, in ascending slot order
            assert bool((es >= 0).all()) and bool((es < B).all())
            if b > 1:
                assert bool((es[:, 1:] > es[:, :-1]).all())
            assert bool((torch.gather(c.pos, 1, es.long()) == (qp0[:, None] + torch.arange(b, device="cuda")[None])).all())
        else:
            assert bool((es == -1).all())
        g_out, g_slot, g_pos = P.to_host(out[sidx]), P.to_host(es[sidx]), P.to_host(ep[sidx])
        for k, u in enumerate(sample):
            ties += P.lockstep_block_unit(states[k], k, g_out, g_slot, g_pos, hQ[k, t:t + b], hK[k, t:t + b],
                                          hV[k, t:t + b], t, s, sc, dtype, what=f"[f32-d64-block] block {i} unit {u}")
        if t >= B or i % 8 == 7:  # cache contents and statistics: every block once full, every eighth while filling
            host = dict(K=P.to_host(c.K[sidx]), V=P.to_host(c.V[sidx]), stats=P.to_host(c.stats[sidx]),
                        pos=P.to_host(c.pos[sidx]), n_used=P.to_host(c.n_used[sidx]))
            for k, u in enumerate(sample):
                P.check_cache_unit(host, k, states[k], what=f"[f32-d64-block] block {i} unit {u}")
        t += b
    print("[f32-d64-block] ties", ties, flush=True)
    P.assert_few_ties(ties, "f32-d64-block")
