"""roco_decode_step_static (the decode step on the library's own static scratch, for callers that cannot allocate)
against roco_decode_step, through the C ABI: two calls in a row, the second on a smaller shape, so that the scratch
still holds the first call's logits and partial results when the second one runs.  Same kernels on another buffer: the
outputs and every piece of cache state must agree bit for bit."""
import ctypes

import numpy as np
import pytest
import torch

from inputs import round_to_bf16

pytestmark = pytest.mark.gpu


def _case(units, L, B, s, d, dtype, steps, seed):
    import parity as P
    rng = np.random.default_rng(seed)
    T = L + steps
    Q = rng.standard_normal((units, T, d)).astype(np.float32) + 0.2
    K = rng.standard_normal((units, T, d)).astype(np.float32)
    V = rng.standard_normal((units, T, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    sess = P.make_session(units, d, B, s, dtype)
    lens = [L - 3 * u for u in range(units)]
    P.gpu_prefill(sess, Q[:, :L].copy(), K[:, :L].copy(), V[:, :L].copy(), lens, False)
    return P, sess, Q, K, V, lens


def _state(c):
    return [t.clone() for t in (c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot)]


def _restore(c, st):
    for t, s in zip((c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot), st):
        t.copy_(s)


def _steps(P, sess, Q, K, V, lens, L, steps, static):
    import paper_2402_06262_amd as roco
    c, p = sess.cache, sess.params
    rec = []
    for t in range(steps):
        dq, dk, dv = (P.to_dev(x[:, L + t], sess.dtype) for x in (Q, K, V))
        qpos = torch.tensor([n + t for n in lens], dtype=torch.int32, device="cuda")
        out = torch.zeros((p.units, p.head_dim), dtype=P.torch_dtype(sess.dtype), device="cuda")
        es = torch.full((p.units,), -7, dtype=torch.int32, device="cuda")
        ep = torch.full((p.units,), -7, dtype=torch.int32, device="cuda")
        if static:
            roco.roco_decode_step_static(p, dq, dk, dv, qpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, out, es, ep)
        else:
            roco.roco_decode_step(p, dq, dk, dv, qpos, c.K, c.V, c.stats, c.pos, c.n_used, c.next_slot, out, es, ep,
                                  sess.decode_ws)
        torch.cuda.synchronize()
        rec.append([out.clone(), es.clone(), ep.clone()] + _state(c))
    return rec


@pytest.mark.parametrize("fused", ["0", "1"])
def test_static_scratch_decode_step_equals_the_workspace_one_on_two_calls_in_a_row(monkeypatch, fused):
    """fused = 0: slot ranges on several workgroups, whose logits and partial results live in the scratch; fused = 1:
    one workgroup per unit (the scratch is then not read, the entry point must still behave the same)."""
    import paper_2402_06262_amd as roco
    monkeypatch.setenv("ROCO_DECODE_FUSED", fused)
    big = dict(units=6, L=700, B=512, s=24, d=128, dtype="bf16", steps=3, seed=201)
    small = dict(units=3, L=140, B=96, s=9, d=64, dtype="f32", steps=3, seed=202)
    for shape in (big, small):  # the second call finds the first one's data in the scratch
        P, sess, Q, K, V, lens = _case(**shape)
        assert roco.decode_workspace_bytes(sess.params) <= 32 << 20
        start = _state(sess.cache)
        want = _steps(P, sess, Q, K, V, lens, shape["L"], shape["steps"], static=False)
        _restore(sess.cache, start)
        torch.cuda.synchronize()
        got = _steps(P, sess, Q, K, V, lens, shape["L"], shape["steps"], static=True)
        for t, (a, b) in enumerate(zip(got, want)):
            for x, y in zip(a, b):
                assert torch.equal(x, y), f"{shape}: step {t} differs between the two entry points"
        assert int(want[-1][1].min()) >= 0  # the steps did evict: the selection ran on the scratch's keys


def test_static_scratch_decode_step_refuses_what_does_not_fit():
    """A shape that needs more than the static 32 MiB is refused on the host, before any launch."""
    import paper_2402_06262_amd as roco
    p = roco.RocoParams(4096, 128, 4096, 64, roco.ROCO_BF16)
    assert roco.decode_workspace_bytes(p) > 32 << 20
    rc = roco.load_library().roco_decode_step_static(ctypes.byref(p), *([0x1000] * 13), None)
    assert rc == -5 and "static" in roco.roco_strerror(rc)
