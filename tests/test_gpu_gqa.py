"""GPU parity of the grouped-query steps (roco_decode_step_gqa, roco_encode_block_gqa) with the oracle."""
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


def empty_states(units, B, d):
    return [orc.CacheState(np.zeros((B, d)), np.zeros((B, d)), np.zeros(B), np.zeros(B), np.zeros(B),
                           np.full(B, -1, dtype=np.int64), 0) for _ in range(units)]


def drive(units, B, s, group, blocks, seed, recency=False, tag="", single_token_entry=False, dtype="bf16", d=128):
    """Key/value heads shared by `group` query heads, encoded from an empty cache in blocks of the given sizes
    (a block of 1 through roco_decode_step_gqa when `single_token_entry`)."""
    import paper_2402_06262_amd as roco
    P = _P()
    sc = 1.0 / math.sqrt(d)
    T = sum(blocks)
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((units, T, group, d)).astype(np.float32) + 0.25
    K = rng.standard_normal((units, T, d)).astype(np.float32)
    V = rng.standard_normal((units, T, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    rw, rb = (24, 0.5) if recency else (0, 0.0)
    sess = P.make_session(units, d, B, s, dtype, 0.0, rw, rb)
    states = empty_states(units, B, d)
    ties = P.TieCount()
    t = 0
    for n_blk, b in enumerate(blocks):
        ws = torch.empty(max(16, roco.block_workspace_bytes(sess.params, b)), dtype=torch.uint8, device="cuda")
        if n_blk % 16 == 0 or b > 1:
            print(f"[{tag}] block of {b} x {group} heads at row {t}", flush=True)
        if b == 1 and single_token_entry:
            o, es, ep = P.gpu_decode_step_gqa(sess, group, Q[:, t], K[:, t], V[:, t], [t] * units, ws)
            g_out, g_slot, g_pos = o[:, None], es[:, None], ep[:, None]
        else:
            g_out, g_slot, g_pos = P.gpu_encode_block_gqa(sess, b, group, Q[:, t:t + b], K[:, t:t + b], V[:, t:t + b],
                                                          [t] * units, ws)
        for u in range(units):
            ties += P.lockstep_block_gqa_unit(states[u], u, g_out, g_slot, g_pos, Q[u, t:t + b], K[u, t:t + b],
                                              V[u, t:t + b], t, s, sc, dtype, rw, rb, what=f"[{tag}] block {b} @ {t}")
        if n_blk % 8 == 7 or n_blk == len(blocks) - 1:
            host = P.cache_to_host(sess)
            for u in range(units):
                P.check_cache_unit(host, u, states[u], what=f"[{tag}] after block {b} @ {t}")
        t += b
    print(f"[{tag}] ties {ties}", flush=True)
    P.assert_few_ties(ties, tag)
    return ties


@pytest.fixture(params=["single", "prepared"])
def single_step(request, monkeypatch):
    """A single-token step books its token inside the attention and finishing kernels; the general block path (a
    preparing kernel first) stays selectable, and both must agree with the oracle."""
    monkeypatch.setenv("ROCO_BLOCK_SINGLE", "0" if request.param == "prepared" else "1")
    return request.param


@pytest.mark.parametrize("group", [1, 2, 4, 8, 32, 64])
def test_grouped_decode_steps_fill_then_evict(group, single_step):
    """Token-wise grouped-query decode from an empty cache: 96 appends, then 40 evicting steps."""
    drive(3, 96, 12, group, [1] * 136, seed=80 + group, tag=f"gqa-decode-g{group}", single_token_entry=True)


@pytest.mark.parametrize("group,blocks", [(4, [8] * 12 + [3, 8, 1, 5, 8]), (2, [16] * 7 + [9, 16]), (3, [10, 7, 10, 10, 2] * 3),
                                          (4, [16] * 3 + [9, 16, 16, 3, 16, 1, 16]), (8, [8] * 7 + [5, 8, 8]), (5, [12, 7, 12] * 4),
                                          (2, [32, 17, 32, 32]), (64, [1] * 70)])
def test_grouped_blocks(group, blocks):
    """Block-wise grouped-query encoding (block * group query rows on one or two matrix tiles), ragged blocks and
    blocks that straddle the budget (B = 64: the cache fills inside the fourth block of 16 tokens) included."""
    drive(2, 64, 8, group, blocks, seed=90 + group, tag=f"gqa-block-g{group}")


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 64)])
def test_grouped_steps_on_the_vector_path(dtype, d):
    """Grouped-query decode and block steps for the shapes that take the vector-ALU attention."""
    drive(2, 48, 6, 4, [1] * 60 + [8, 3, 8, 1, 16, 11, 16], seed=170 + d, tag=f"gqa-simple-{dtype}-{d}", single_token_entry=True,
          dtype=dtype, d=d)


def test_grouped_steps_with_recency_bias_and_a_larger_budget(single_step):
    drive(2, 1024, 48, 4, [8] * 130 + [1] * 8, seed=97, recency=True, tag="gqa-recency", single_token_entry=True)


def run_grouped_prefill(dtype, d, group, lens, L, B, s, seed, steps=6, recency=False, policy=None, tag="",
                        want_out=True):
    """roco_prefill_compress_gqa against the oracle, then grouped decode steps from the compressed caches."""
    import paper_2402_06262_amd as roco
    P = _P()
    units = len(lens)
    sc = 1.0 / math.sqrt(d)
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((units, group, L + steps, d)).astype(np.float32) + 0.25
    K = rng.standard_normal((units, L + steps, d)).astype(np.float32)
    V = rng.standard_normal((units, L + steps, d)).astype(np.float32)
    heavy = rng.choice(L, size=max(1, L // 40), replace=False)
    K[:, heavy] += 2.0
    if dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    rw, rb = (24, 0.5) if recency else (0, 0.0)
    sess = P.make_session(units, d, B, s, dtype, 0.0, rw, rb, policy=policy)
    print(f"[{tag}] grouped prefill {dtype} d={d} g={group} lens={lens} B={B}", flush=True)
    g_res = P.gpu_prefill_gqa(sess, group, Q[:, :, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), lens, want_out)
    ties = P.TieCount()
    states = []
    for u in range(units):
        full = orc.prefill_statistics_gqa(Q[u, :, :L], K[u, :L], V[u, :L], lens[u], sc, rw, rb, policy=policy,
                                          want_out=want_out)
        res, t = P.check_prefill_unit(g_res, u, None, K[u, :L], V[u, :L], lens[u], B, s, sc, dtype, rw, rb, False,
                                      full=full, policy=policy)
        if want_out:  # the attention output of every head and prompt row
            for h in range(group):
                for i in range(lens[u]):
                    P.assert_out_close(g_res["O"][u, h, i], full.out[h, i], dtype, f"[{tag}] unit {u} head {h} O[{i}]")
        ties += t
        states.append(res.cache)
    ws = torch.empty(roco.block_workspace_bytes(sess.params, 1), dtype=torch.uint8, device="cuda")
    nxt = list(lens)
    for i in range(steps):
        t = L + i
        o, es, ep = P.gpu_decode_step_gqa(sess, group, Q[:, :, t], K[:, t], V[:, t], nxt, ws)
        for u in range(units):
            ties += P.lockstep_block_gqa_unit(states[u], u, o[:, None], es[:, None], ep[:, None], Q[u, :, t][None],
                                              K[u, t:t + 1], V[u, t:t + 1], nxt[u], s, sc, dtype, rw, rb,
                                              what=f"[{tag}] step {i}")
        nxt = [x + 1 for x in nxt]
    host = P.cache_to_host(sess)
    for u in range(units):
        P.check_cache_unit(host, u, states[u], what=f"[{tag}] end")
    print(f"[{tag}] ties {ties}", flush=True)
    P.assert_few_ties(ties, tag)


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128), ("bf16", 64)])
@pytest.mark.parametrize("group", [1, 2, 4])
def test_grouped_prefill_then_grouped_decode(dtype, d, group):
    run_grouped_prefill(dtype, d, group, [300, 257, 130, 60], 300, 128, 14, seed=500 + group + d,
                        tag=f"gqa-prefill-{dtype}-{d}-g{group}")


@pytest.mark.parametrize("group", [2, 4, 8, 16])
@pytest.mark.parametrize("recency", [False, True])
@pytest.mark.parametrize("ring", ["ring", "staged"])
def test_grouped_prefill_on_the_matrix_cores_with_heads_summed_in_registers(group, recency, ring, monkeypatch):
    """Group sizes that divide 16 take the column pass whose tiles hold all heads of a few query positions: lengths
    around its tile edges (64 / g positions per tile), several key blocks, with and without the recency bias; the
    query tiles of a key block on one workgroup (as with many units) or shared by two (as with few); tiles fed by the
    LDS ring (the default) or staged through registers."""
    monkeypatch.setenv("ROCO_PREFILL_QSPLIT", "1" if recency else "2")
    monkeypatch.setenv("ROCO_PREFILL_GQA_RING", "1" if ring == "ring" else "0")
    run_grouped_prefill("bf16", 128, group, [517, 300, 64 // group + 1, 129, 33], 517, 100, 12, seed=540 + group,
                        recency=recency, tag=f"gqa-pow2-g{group}-{recency}-{ring}", steps=2)


@pytest.mark.parametrize("group", [2, 4, 16])
def test_grouped_prefill_long_prompts_through_the_ring(group):
    """Prompts of many key blocks and query tiles: the rectangle of the ring-fed grouped column pass (software-pipelined,
    head sums carried across its slices) does most of the work; ragged lengths, one prompt shorter than the budget."""
    run_grouped_prefill("bf16", 128, group, [1500, 1337, 1024, 90], 1500, 256, 40, seed=560 + group,
                        tag=f"gqa-ring-long-g{group}", steps=2)


def test_grouped_prefill_with_eight_heads_under_the_accumulated_score():
    """Several key blocks per unit, two units, eight heads, ranked by the accumulated score over the whole cache."""
    run_grouped_prefill("bf16", 128, 8, [700, 420], 700, 256, 256, seed=551, policy=orc.Policy("aas", "all"),
                        tag="gqa-pow2-aas", steps=0)


def test_grouped_prefill_with_recency_bias_and_three_heads():
    run_grouped_prefill("bf16", 128, 3, [200, 77], 200, 64, 9, seed=520, recency=True, tag="gqa-prefill-recency")


def test_grouped_prefill_under_the_last_token_score():
    run_grouped_prefill("bf16", 128, 4, [260, 150], 260, 96, 96, seed=530, policy=orc.Policy("ltas", "all"),
                        tag="gqa-prefill-ltas", steps=0)


@pytest.mark.timeout(600)
def test_grouped_prefill_at_the_serving_shape():
    """128 key/value heads x 4 query heads (batch 16 x 8), prompt 3072 -> B = 2048, scope 64: every unit on the GPU,
    properties on all of them, the oracle on a sample."""
    import paper_2402_06262_amd as roco
    P = _P()
    U, g, d, L, B, s = 128, 4, 128, 3072, 2048, 64
    sc = 1.0 / math.sqrt(d)
    rng = np.random.default_rng(777)
    sample = [0, 101]
    dt = torch.bfloat16
    dQ = torch.empty((U, g, L, d), dtype=dt, device="cuda")
    dK = torch.empty((U, L, d), dtype=dt, device="cuda")
    dV = torch.empty_like(dK)
    host = {}
    for u in range(U):
        q = rng.standard_normal((g, L, d), dtype=np.float32) + 0.25
        k = rng.standard_normal((L, d), dtype=np.float32)
        v = rng.standard_normal((L, d), dtype=np.float32)
        k[rng.choice(L, size=60, replace=False)] += 1.5
        dQ[u], dK[u], dV[u] = (torch.from_numpy(x).cuda().to(dt) for x in (q, k, v))
        if u in sample:
            host[u] = tuple(t.float().cpu().numpy() for t in (dQ[u], dK[u], dV[u]))
    sess = P.make_session(U, d, B, s, "bf16")
    c, p = sess.cache, sess.params
    ws = torch.empty(roco.prefill_gqa_workspace_bytes(p, g, L), dtype=torch.uint8, device="cuda")
    dlen = torch.full((U,), L, dtype=torch.int32, device="cuda")
    print("[gqa-prefill-serving] prefill", flush=True)
    roco.roco_prefill_compress_gqa(p, g, dQ, dK, dV, dlen, L, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, None, ws)
    torch.cuda.synchronize()
    pos = c.pos.long()
    assert bool((c.n_used == B).all()) and bool((pos[:, 1:] > pos[:, :-1]).all()) and int(pos.min()) >= 0 and int(pos.max()) < L
    assert bool((c.stats[:, 2] == (L - pos).float()).all())
    idx = pos[:, :, None].expand(U, B, d)
    assert torch.equal(torch.gather(dK, 1, idx), c.K) and torch.equal(torch.gather(dV, 1, idx), c.V)
    assert bool((c.next_slot >= 0).all()) and bool((c.next_slot < B).all())
    sidx = torch.tensor(sample, device="cuda")
    g_res = dict(K=P.to_host(c.K[sidx]), V=P.to_host(c.V[sidx]), stats=P.to_host(c.stats[sidx]),
                 pos=P.to_host(c.pos[sidx]), n_used=P.to_host(c.n_used[sidx]), O=None)
    ties = P.TieCount()
    for k_, u in enumerate(sample):
        Qh, Kh, Vh = host[u]
        print(f"[gqa-prefill-serving] oracle statistics of unit {u}", flush=True)
        full = orc.prefill_statistics_gqa(Qh, Kh, Vh, L, sc)
        _, t = P.check_prefill_unit(g_res, k_, None, Kh, Vh, L, B, s, sc, "bf16", 0, 0.0, False, full=full)
        ties += t
    print(f"[gqa-prefill-serving] ties {ties}", flush=True)
    P.assert_few_ties(ties, "gqa-prefill-serving")


def test_grouped_decode_at_the_serving_shape():
    """The shape bench.py times for g = 4: 128 key/value heads (batch 16 x 8), B = 2048, scope 64, full cache.
    All units step on the GPU; properties on every unit, the oracle in lock-step on a sample."""
    import paper_2402_06262_amd as roco
    P = _P()
    U, B, s, g, d, L, steps = 128, 2048, 64, 4, 128, 2100, 6
    sc = 1.0 / math.sqrt(d)
    rng = np.random.default_rng(123)
    sample = [0, 57, 127]
    Qp = round_to_bf16(rng.standard_normal((U, L, d)).astype(np.float32) + 0.25)
    K = round_to_bf16(rng.standard_normal((U, L + steps, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((U, L + steps, d)).astype(np.float32))
    Qg = round_to_bf16(rng.standard_normal((U, steps, g, d)).astype(np.float32) + 0.25)
    sess = P.make_session(U, d, B, s, "bf16")
    gp = P.gpu_prefill(sess, Qp, K[:, :L].copy(), V[:, :L].copy(), [L] * U, False)  # a valid full cache to start from
    states = {u: P.check_prefill_unit(gp, u, Qp[u], K[u, :L], V[u, :L], L, B, s, sc, "bf16", 0, 0.0, False)[0].cache
              for u in sample}
    ws = torch.empty(roco.block_workspace_bytes(sess.params, 1), dtype=torch.uint8, device="cuda")
    ties = P.TieCount()
    for i in range(steps):
        t = L + i
        acc_before = sess.cache.stats[:, 0].double().sum(1)
        o, es, ep = P.gpu_decode_step_gqa(sess, g, Qg[:, i], K[:, t], V[:, t], [t] * U, ws)
        assert np.all(es >= 0) and np.all(es < B) and np.isfinite(o).all()
        c = sess.cache
        assert bool((torch.gather(c.pos, 1, torch.from_numpy(es).cuda().long()[:, None])[:, 0] == t).all())
        for u in sample:
            victim_acc = states[u].acc[int(es[u])]
            ties += P.lockstep_block_gqa_unit(states[u], u, o[:, None], es[:, None], ep[:, None], Qg[u, i][None],
                                              K[u, t:t + 1], V[u, t:t + 1], t, s, sc, "bf16", what=f"[gqa-serving] step {i}")
            inc = float(c.stats[u, 0].double().sum() - acc_before[u]) + victim_acc
            assert abs(inc - 1.0) < 2e-3  # the head-mean probabilities of a step sum to one
    host = P.cache_to_host(sess)
    for u in sample:
        P.check_cache_unit({k: v[[u]] for k, v in host.items()}, 0, states[u], what="[gqa-serving] end")
    print(f"[gqa-serving] ties {ties}", flush=True)
    P.assert_few_ties(ties, "gqa-serving")


def test_group_of_one_matches_the_token_wise_decode_step_bit_for_bit_in_its_decisions():
    """roco_decode_step_gqa with one head and roco_decode_step on identical inputs: same victims, same positions;
    statistics and outputs within the parity tolerances (different kernels, different summation order)."""
    import paper_2402_06262_amd as roco
    P = _P()
    units, B, s, d = 4, 128, 16, 128
    rng = np.random.default_rng(99)
    T = B + 48
    Q = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32) + 0.25)
    K = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    a = P.make_session(units, d, B, s, "bf16")
    b = P.make_session(units, d, B, s, "bf16")
    ws = torch.empty(roco.block_workspace_bytes(b.params, 1), dtype=torch.uint8, device="cuda")
    for t in range(T):
        o1, s1, p1 = P.gpu_decode_step(a, Q[:, t], K[:, t], V[:, t], [t] * units)
        o2, s2, p2 = P.gpu_decode_step_gqa(b, 1, Q[:, t, None], K[:, t], V[:, t], [t] * units, ws)
        assert np.array_equal(p1, p2), f"step {t}: evicted positions differ"
        assert np.array_equal(s1, s2), f"step {t}: evicted slots differ"
        for u in range(units):
            P.assert_out_close(o2[u, 0], o1[u].astype(np.float64), "bf16", f"step {t} unit {u}")
    ha, hb = P.cache_to_host(a), P.cache_to_host(b)
    assert np.array_equal(ha["pos"], hb["pos"]) and np.array_equal(ha["stats"][:, 2], hb["stats"][:, 2])
    P.assert_stat_close(hb["stats"][:, 0], ha["stats"][:, 0].astype(np.float64), "Acc")


def test_grouped_and_block_steps_captured_in_a_hip_graph_replay_like_eager_steps():
    """The block-wise and grouped steps allocate nothing and never synchronise either.  A grouped single-token step,
    a grouped block and another single-token step are captured once and replayed three times with eager work and
    synchronisations in between; every replay must leave exactly what the same calls leave when launched eagerly."""
    import paper_2402_06262_amd as roco
    import test_gpu_parity as TP
    P = _P()
    units, L, B, s, d, g, b = 5, 180, 96, 12, 128, 4, 6
    rng = np.random.default_rng(77)
    T = L + 2 + b
    Q = round_to_bf16(rng.standard_normal((units, g, T, d)).astype(np.float32) + 0.2)
    K = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    V = round_to_bf16(rng.standard_normal((units, T, d)).astype(np.float32))
    sess = P.make_session(units, d, B, s, "bf16")
    P.gpu_prefill_gqa(sess, g, Q[:, :, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), [L, L, 150, 96, 40], False)
    c, p = sess.cache, sess.params
    ws = torch.empty(roco.block_workspace_bytes(p, b), dtype=torch.uint8, device="cuda")
    dev = lambda x: P.to_dev(np.ascontiguousarray(x), "bf16")
    lens = torch.tensor([L, L, 150, 96, 40], dtype=torch.int32, device="cuda")
    q1, k1, v1 = dev(Q[:, :, L]), dev(K[:, L]), dev(V[:, L])
    qb, kb, vb = dev(Q[:, :, L + 1:L + 1 + b].transpose(0, 2, 1, 3)), dev(K[:, L + 1:L + 1 + b]), dev(V[:, L + 1:L + 1 + b])
    q2, k2, v2 = dev(Q[:, :, T - 1]), dev(K[:, T - 1]), dev(V[:, T - 1])
    pos1, posb, pos2 = lens.clone(), lens + 1, lens + 1 + b
    o1 = torch.zeros((units, g, d), dtype=torch.bfloat16, device="cuda")
    ob = torch.zeros((units, b, g, d), dtype=torch.bfloat16, device="cuda")
    o2 = torch.zeros_like(o1)
    e1 = torch.zeros((units,), dtype=torch.int32, device="cuda")
    eb = torch.zeros((units, b), dtype=torch.int32, device="cuda")
    e2 = torch.zeros_like(e1)

    def run_steps():
        roco.roco_decode_step_gqa(p, g, q1, k1, v1, pos1, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, o1, e1, None, ws)
        roco.roco_encode_block_gqa(p, b, g, qb, kb, vb, posb, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, ob, eb,
                                   None, ws)
        roco.roco_decode_step_gqa(p, g, q2, k2, v2, pos2, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, o2, e2, None, ws)

    def snapshot():
        return [x.clone() for x in (o1, ob, o2, e1, eb, e2)] + TP._state(c)

    start = TP._state(c)
    want = []
    for _ in range(3):  # the state keeps evolving from round to round (positions repeat; only equality matters here)
        run_steps()
        torch.cuda.synchronize()
        want.append(snapshot())
    TP._restore(c, start)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_steps()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    TP._restore(c, start)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_steps()
    TP._restore(c, start)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device="cuda")
    for r in range(3):
        graph.replay()
        scratch.add_(1.0)
        torch.cuda.synchronize()
        for a, w in zip(snapshot(), want[r]):
            assert torch.equal(a, w), f"replay {r} differs from the eager calls"
