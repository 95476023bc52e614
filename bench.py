#!/usr/bin/env python3
"""Benchmark of the RoCo hot path on one MI355X.

One *step* is one pass of the whole path over one batch of the serving workload (workload 3: one 32-head x
128-dim bf16 layer, batch 16): prefill-compress of the 3072-token prompts to B = 2048 with scope 64, then
`--decode-steps` (default 512) decode steps, each appending one token and evicting one slot per head.
Inputs are seeded synthetic heavy-hitter Q/K/V, resident in HBM before the timed region.

Prints ONE JSON line: `value` is decode tokens/s (batch x decode steps / decode time); prefill+evict tokens/s,
the HBM roofline of the dominant decode kernel, the MFMA roofline of the prefill statistics kernels and the
CPU oracle timed on this machine's host cores ride along in the same line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix peak
ALU_SLOTS_PER_MFMA = {"rows": 9, "columns": 11}  # issue slots per matrix instruction, see alu_cobound_tflops


def alu_cobound_tflops(which):
    """What the vector ALU allows the prefill passes, as a matrix rate.  A 32x32x16 matrix instruction produces two
    scores per lane and occupies the matrix pipe of its SIMD for 32 cycles; a SIMD issues one vector instruction of a
    wave per 4 cycles (64 lanes on 16 lanes per clock: 64 fp32 lanes per clock and compute unit), and the exponential
    takes two such slots.  Per score the row pass needs multiply-add + exponential + add = 4 slots, the column pass
    one multiply-add more = 5; with the matrix instruction's own slot that is 9 / 11 slots = 36 / 44 cycles per matrix
    instruction against 32: 0.89 / 0.73 of the matrix peak, however the two kinds are interleaved."""
    return MFMA_BF16_PEAK_TFLOPS * 32.0 / (4.0 * ALU_SLOTS_PER_MFMA[which])


def measured_traffic(kernel, workload):
    """HBM-side bytes per launch of `kernel` on `workload`, as rocprofv3 counted them: the TRAFFIC lines of the
    summaries under profiles/ (each names the kernel, the workload and the commit it was measured at).  None when no
    line matches: the figure is never carried over to another kernel or shape."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        with open(path) as f:
            for line in f:
                if not line.startswith("TRAFFIC "):
                    continue
                rec = dict(kv.split("=", 1) for kv in line.split()[1:])
                if rec.get("kernel") == kernel and rec.get("workload") == str(workload):
                    return {"bytes": int(rec["fetch_bytes"]) + int(rec["write_bytes"]), "fetch_bytes": int(rec["fetch_bytes"]),
                            "write_bytes": int(rec["write_bytes"]), "kernel": kernel, "measured_at_commit": rec.get("commit"),
                            "source": os.path.relpath(path, ROOT)}
    return None


def counted_issue_bound_tflops(kernel, workload):
    """The matrix rate at which the vector-issue port saturates with the instruction mix rocprofv3 counted for
    `kernel` (COUNTED lines under profiles/): per matrix instruction its own issue slot, one per vector instruction
    and a second one per transcendental, 4 cycles each, against the pipe's 32 cycles.  None without a counted mix."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        with open(path) as f:
            for line in f:
                if line.startswith("COUNTED "):
                    rec = dict(kv.split("=", 1) for kv in line.split()[1:])
                    if rec.get("kernel") == kernel and rec.get("workload") == str(workload):
                        slots = 1.0 + float(rec["valu_per_mfma"]) + float(rec["trans_per_mfma"])
                        return {"TFLOPs": MFMA_BF16_PEAK_TFLOPS * 32.0 / (4.0 * slots), "issue_slots_per_mfma": slots,
                                "measured_at_commit": rec.get("commit"), "source": os.path.relpath(path, ROOT)}
    return None


def generate(cfg, seed, workers):
    """All units of the workload as float32 host arrays [units, T, d] (bf16-representable)."""
    from inputs import make_unit, unit_ids
    ids = unit_ids(cfg)
    T, d = cfg.total_len, cfg.head_dim
    Q = np.empty((len(ids), T, d), np.float32)
    K = np.empty_like(Q)
    V = np.empty_like(Q)

    def one(i):
        u = make_unit(cfg, *ids[i], seed=seed)
        Q[i], K[i], V[i] = u.Q, u.K, u.V

    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(one, range(len(ids))))
    return Q, K, V


def upload(x, torch, dt, chunk=64):
    out = torch.empty(x.shape, dtype=dt, device="cuda")
    for i in range(0, x.shape[0], chunk):
        out[i:i + chunk] = torch.from_numpy(x[i:i + chunk]).cuda().to(dt)
    return out


def cpu_baseline(cfg, Q, K, V, decode_steps, n_units, n_steps):
    """The float64 oracle, as it stands, on a bounded sample of this workload's units."""
    from oracle import roco_oracle as orc
    L, B, s = cfg.prompt_len, cfg.budget, cfg.scope
    sc = 1.0 / math.sqrt(cfg.head_dim)
    n_steps = min(n_steps, decode_steps)
    t0 = time.perf_counter()
    states = []
    for u in range(n_units):
        states.append(orc.prefill_compress(Q[u, :L], K[u, :L], V[u, :L], L, B, s, sc).cache)
    t1 = time.perf_counter()
    for u in range(n_units):
        for t in range(L, L + n_steps):
            orc.decode_step(states[u], Q[u, t], K[u, t], V[u, t], t, s, sc)
    t2 = time.perf_counter()
    per_unit_prefill = (t1 - t0) / n_units
    per_unit_step = (t2 - t1) / max(1, n_units * n_steps)
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    return {
        "value": cfg.batch / (cfg.units * per_unit_step) if per_unit_step > 0 else None,
        "unit": "tokens/s",
        "prefill_evict_tokens_per_s": cfg.batch * L / (cfg.units * per_unit_prefill),
        "cores": int(threads),
        "host_cores_visible": len(os.sched_getaffinity(0)),
        "kind": "oracle",
        "sample": f"float64 NumPy oracle on units 0..{n_units - 1} of {cfg.units}: prefill-compress {L}->{B}, then "
                  f"{n_steps} decode steps each; scaled linearly to {cfg.units} units "
                  f"({t2 - t0:.1f} s of CPU work)",
    }


def _decode_loop(torch, roco, p, cache, sq, sk, sv, qpos, out, ev_slot, ev_pos, ws, stream):
    """A function that runs all decode steps of [steps, units, d] inputs through roco_decode_step (addresses worked out
    once, plain integers into the C entry point: the loop is launch-rate sensitive)."""
    import ctypes
    lib = roco.load_library()
    steps, U, d = sq.shape
    esz = sq.element_size()
    row = U * d * esz
    pref = ctypes.byref(p)
    c = [x.data_ptr() for x in (cache.K, cache.V, cache.stats, cache.pos, cache.n_used, cache.next_slot)]
    args = [(sq.data_ptr() + t * row, sk.data_ptr() + t * row, sv.data_ptr() + t * row, qpos.data_ptr() + t * U * 4)
            for t in range(steps)]
    o, es, ep, w, wb, st = out.data_ptr(), ev_slot.data_ptr(), ev_pos.data_ptr(), ws.data_ptr(), ws.numel(), stream.cuda_stream

    def run():
        for a in args:
            rc = lib.roco_decode_step(pref, a[0], a[1], a[2], a[3], c[0], c[1], c[2], c[3], c[4], c[5], o, es, ep, w, wb, st)
            if rc != 0:
                raise roco.RocoError(rc, "roco_decode_step")
    return run


def _timed(torch, stream, fn, reps=1):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def side_workloads(torch, roco, seed, which):
    """Throughput of the other benchmark workloads (1, 2, 4, 5), each with the roofline that bounds it: MFMA for the
    prompt passes, HBM for the decode step where the step's working set is far larger than the 256 MB last-level cache
    (workload 4), no bandwidth claim where it fits (workload 5) or where a step is launch latency (workload 1)."""
    from inputs import CONFIGS, make_unit, unit_ids
    from inputs.device import make_layer_on_device
    stream = torch.cuda.current_stream()
    res = {}
    for idx in which:
        cfg = CONFIGS[idx - 1]
        L, B, s, d, steps = cfg.prompt_len, cfg.budget, cfg.scope, cfg.head_dim, cfg.steps
        dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        esz = 2 if cfg.dtype == "bf16" else 4
        rdt = roco.ROCO_BF16 if cfg.dtype == "bf16" else roco.ROCO_F32
        per_layer = cfg.batch * cfg.heads
        U = cfg.units
        p = roco.RocoParams(U, d, B, s, rdt, 0.0, cfg.recency_window, cfg.recency_bias)
        lp = roco.RocoParams(per_layer, d, B, s, rdt, 0.0, cfg.recency_window, cfg.recency_bias)
        cache = roco.alloc_cache(p)
        ws_p = torch.empty(roco.prefill_workspace_bytes(lp, L), dtype=torch.uint8, device="cuda")
        dlen = torch.full((per_layer,), L, dtype=torch.int32, device="cuda")
        sq = torch.empty((max(steps, 1), U, d), dtype=dt, device="cuda")
        sk, sv = torch.empty_like(sq), torch.empty_like(sq)
        prefill_ms = 0.0
        for layer in range(cfg.layers):  # the prompt pass runs layer by layer, as a model would call it
            if idx >= 4:  # drawn on the device: the host generator would need minutes
                Qd, Kd, Vd, _ = make_layer_on_device(cfg, layer, seed=seed)
            else:
                units = [make_unit(cfg, *i, seed=seed) for i in unit_ids(cfg)]
                Qd, Kd, Vd = (upload(np.stack([getattr(u_, n_) for u_ in units]), torch, dt) for n_ in ("Q", "K", "V"))
            lo, hi = layer * per_layer, (layer + 1) * per_layer
            dQ, dK, dV = (x[:, :L].contiguous() for x in (Qd, Kd, Vd))
            if steps:
                for x, dst in ((Qd, sq), (Kd, sk), (Vd, sv)):
                    dst[:, lo:hi] = x[:, L:L + steps].transpose(0, 1)
            del Qd, Kd, Vd

            def prefill():
                roco.roco_prefill_compress(lp, dQ, dK, dV, dlen, L, cache.K[lo:hi], cache.V[lo:hi], cache.stats[lo:hi],
                                           cache.pos[lo:hi], cache.n_used[lo:hi], cache.next_slot[lo:hi], None, ws_p, stream=stream)
            prefill()  # warm-up
            torch.cuda.synchronize()
            prefill_ms += _timed(torch, stream, prefill, 3 if cfg.layers > 1 else 5)
            del dQ, dK, dV
        flops = U * 2 * d * L * (L + 1)
        tf = flops / (prefill_ms * 1e-3) / 1e12
        r = {"workload": f"config {idx}: {cfg.layers} layer(s) x batch {cfg.batch} x {cfg.heads} heads x {d} dims {cfg.dtype}, "
                         f"prompt {L} -> B={B}, scope {s}, {steps} decode steps", "units": U,
             "prefill_ms": prefill_ms, "prefill_evict_tokens_per_s": cfg.batch * L / (prefill_ms * 1e-3)}
        if cfg.dtype == "bf16" and d == 128:
            r["roofline_prefill"] = {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": tf / MFMA_BF16_PEAK_TFLOPS, "flops": flops}
        else:
            r["roofline_prefill"] = {"bound": "alu", "achieved": tf, "peak": None, "unit": "TFLOP/s", "frac": None,
                                     "note": "fp32 / head_dim 64 takes the vector-ALU passes; 4 units: latency, no claim"}
        if steps:
            qpos = (torch.arange(steps, dtype=torch.int32, device="cuda")[:, None] + L).expand(steps, U).contiguous()
            out = torch.empty((U, d), dtype=dt, device="cuda")
            ev_slot = torch.empty((U,), dtype=torch.int32, device="cuda")
            ev_pos = torch.empty_like(ev_slot)
            snap = [t.clone() for t in (cache.K, cache.V, cache.stats, cache.pos, cache.n_used, cache.next_slot)]
            step_bytes = U * B * (2 * d * esz + 24)
            by_scope = {}
            for scope in (cfg.scope_sweep or (s,)):
                ps = roco.RocoParams(U, d, B, scope, rdt, 0.0, cfg.recency_window, cfg.recency_bias)
                ws_d = torch.empty(max(16, roco.decode_workspace_bytes(ps)), dtype=torch.uint8, device="cuda")
                run = _decode_loop(torch, roco, ps, cache, sq, sk, sv, qpos, out, ev_slot, ev_pos, ws_d, stream)
                best = None
                for rep in range(2):
                    for t, sn in zip((cache.K, cache.V, cache.stats, cache.pos, cache.n_used, cache.next_slot), snap):
                        t.copy_(sn)
                    if scope != s:
                        roco.roco_select_victims(ps, cache.stats, cache.pos, cache.n_used, cache.next_slot, ws_d, stream=stream)
                    torch.cuda.synchronize()
                    ms = _timed(torch, stream, run)
                    best = ms if best is None else min(best, ms)
                assert int(cache.n_used.min()) == B and int((ev_slot >= 0).sum()) == U
                by_scope[str(scope)] = {"ms_per_token_step": best / steps, "tokens_per_s": cfg.batch * steps / (best * 1e-3),
                                        "step_GBps": step_bytes / (best * 1e-3 / steps) / 1e9,
                                        "launches_per_step": roco.decode_step_launches(ps)}
                del ws_d
            main_scope = by_scope[str(s)]
            r["decode_ms_per_token_step"] = main_scope["ms_per_token_step"]
            r["decode_tokens_per_s"] = main_scope["tokens_per_s"]
            if len(by_scope) > 1:
                r["decode_by_scope"] = by_scope
            cache_bytes = U * B * 2 * d * esz
            if cache_bytes > (1 << 30):  # far beyond the last-level cache: an HBM figure means something
                r["roofline_decode_step"] = {"bound": "hbm", "achieved": main_scope["step_GBps"], "peak": HBM_PEAK_GBS,
                                             "unit": "GB/s", "frac": main_scope["step_GBps"] / HBM_PEAK_GBS,
                                             "bytes_per_step": step_bytes}
            else:
                why = ("fits the 256 MB last-level cache: no HBM claim" if cache_bytes > (8 << 20)
                       else "a step is launch latency: no bandwidth claim")
                r["roofline_decode_step"] = {"bound": "hbm", "achieved": main_scope["step_GBps"], "peak": HBM_PEAK_GBS,
                                             "unit": "GB/s", "frac": None, "bytes_per_step": step_bytes,
                                             "note": f"{cache_bytes / 2**20:.1f} MiB of K and V per step {why}"}
            del snap, qpos
        res[str(idx)] = r
        del cache, ws_p, sq, sk, sv
        torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--decode-steps", type=int, default=None, help="decode steps per pass (default: the workload's 512)")
    ap.add_argument("--seed", type=int, default=20240206)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-units", type=int, default=96)
    ap.add_argument("--cpu-steps", type=int, default=512)
    ap.add_argument("--with-out", action="store_true", help="also produce the prefill attention output O")
    ap.add_argument("--no-blockwise", action="store_true", help="skip the block-wise evict-and-encode table")
    ap.add_argument("--block-sizes", default="1,2,4,8,16,32,64", help="block sizes of the block-wise table")
    ap.add_argument("--gqa-groups", default="1,4,8", help="group sizes of the grouped-query table")
    ap.add_argument("--gqa-block-sizes", default="1,2,4,8,16", help="block sizes encoded with a group of 4")
    ap.add_argument("--no-two-streams", action="store_true",
                    help="skip the decode loop with the batch split over two HIP streams")
    ap.add_argument("--no-consistency", action="store_true", help="skip the synthetic consistency study")
    ap.add_argument("--workloads", default="1,2,4,5",
                    help="the other benchmark workloads to time beside the headline one (comma separated; '' = none)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 512 MiB device copy (a kernel of known traffic, to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; units (layer x sequence x head) are independent and would be "
              "sharded without any collective, but no multi-GPU path exists. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2402_06262_amd as roco
    from inputs import CONFIGS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = CONFIGS[2]
    decode_steps = cfg.steps if args.decode_steps is None else min(cfg.steps, args.decode_steps)
    L, B, s, d, U = cfg.prompt_len, cfg.budget, cfg.scope, cfg.head_dim, cfg.units
    dt = torch.bfloat16
    esz = 2

    t_gen = time.perf_counter()
    Q, K, V = generate(cfg, args.seed, workers=min(16, len(os.sched_getaffinity(0))))
    t_gen = time.perf_counter() - t_gen
    dQ, dK, dV = (upload(x[:, :L], torch, dt) for x in (Q, K, V))
    # per-step decode inputs, [steps, units, d]
    sq, sk, sv = (upload(np.ascontiguousarray(x[:, L:L + decode_steps].transpose(1, 0, 2)), torch, dt)
                  for x in (Q, K, V))
    qpos = (torch.arange(decode_steps, dtype=torch.int32, device="cuda")[:, None] + L).expand(decode_steps, U).contiguous()
    dlen = torch.full((U,), L, dtype=torch.int32, device="cuda")

    p = roco.RocoParams(U, d, B, s, roco.ROCO_BF16)
    cache = roco.alloc_cache(p)
    ws_p = torch.empty(roco.prefill_workspace_bytes(p, L), dtype=torch.uint8, device="cuda")
    ws_d = torch.empty(roco.decode_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    out = torch.empty((decode_steps, U, d), dtype=dt, device="cuda")
    ev_slot = torch.empty((decode_steps, U), dtype=torch.int32, device="cuda")
    ev_pos = torch.empty_like(ev_slot)
    O = torch.empty_like(dQ) if args.with_out else None
    stream = torch.cuda.current_stream()

    def prefill():
        roco.roco_prefill_compress(p, dQ, dK, dV, dlen, L, cache.K, cache.V, cache.stats, cache.pos, cache.n_used,
                                   cache.next_slot, O, ws_p, stream=stream)

    # The decode loop is launch-rate sensitive (a step is ~0.12 ms of GPU time), so the per-step device addresses are
    # worked out once and the C entry point is called with plain integers: no tensor slicing inside the loop.
    import ctypes
    lib = roco.load_library()
    pref = ctypes.byref(p)
    row = U * d * esz
    step_args = [(sq.data_ptr() + t * row, sk.data_ptr() + t * row, sv.data_ptr() + t * row,
                  qpos.data_ptr() + t * U * 4, out.data_ptr() + t * row, ev_slot.data_ptr() + t * U * 4,
                  ev_pos.data_ptr() + t * U * 4) for t in range(decode_steps)]
    cK, cV, cS, cP, cN, cX = (x.data_ptr() for x in (cache.K, cache.V, cache.stats, cache.pos, cache.n_used,
                                                     cache.next_slot))
    wsd_ptr, wsd_bytes, stream_ptr = ws_d.data_ptr(), ws_d.numel(), stream.cuda_stream

    def decode_one(t):
        a = step_args[t]
        rc = lib.roco_decode_step(pref, a[0], a[1], a[2], a[3], cK, cV, cS, cP, cN, cX, a[4], a[5], a[6], wsd_ptr,
                                  wsd_bytes, stream_ptr)
        if rc != 0:
            raise roco.RocoError(rc, "roco_decode_step")

    def decode():
        for t in range(decode_steps):
            decode_one(t)

    for _ in range(args.warmup):
        prefill()
        decode()
    torch.cuda.synchronize()
    if args.calibration_copy:
        src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 512 MiB, writes 512 MiB
        torch.cuda.synchronize()
        del src, dst

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    roco.roco_profile_read()
    roco.roco_profile_sampling(8)  # HIP events around every 8th decode_attend launch of the timed region
    roco.roco_profile_kernel(roco.PROF_KERNELS["decode_attend"])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        ev[k][0].record(stream)
        prefill()
        ev[k][1].record(stream)
        decode()
        ev[k][2].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    attend_ms, attend_n = roco.roco_profile_read()
    roco.roco_profile_kernel(-1)
    roco.roco_profile_sampling(1)

    prefill_ms = sum(e[0].elapsed_time(e[1]) for e in ev)
    decode_ms = sum(e[1].elapsed_time(e[2]) for e in ev)
    decode_tok_s = cfg.batch * decode_steps * args.steps / (decode_ms * 1e-3)
    prefill_tok_s = cfg.batch * L * args.steps / (prefill_ms * 1e-3)

    # sanity on the final state (not a parity test): every unit full, one eviction per unit per step
    assert int(cache.n_used.min()) == B and int(cache.n_used.max()) == B
    assert int((ev_slot >= 0).sum()) == decode_steps * U

    # dominant kernel.  Split path: decode_attend reads every cached K and V element once.  Fused path (one
    # workgroup per unit): decode_fused is the whole step: K and V once, the three statistics read and written.
    fused = roco.decode_step_launches(p) == 1
    step_bytes = U * B * (2 * d * esz + 24)
    attend_bytes = step_bytes if fused else U * B * 2 * d * esz
    attend_name = "decode_fused" if fused else "decode_attend"
    traffic = measured_traffic(attend_name, 3) if (U == 512 and decode_steps > 0) else None
    attend_avg_s = attend_ms * 1e-3 / max(1, attend_n)
    # prefill statistics: two causal QK^T passes (row normalisers, then column statistics), 2 flops per MAC
    prefill_flops = U * 2 * d * L * (L + 1) * (1.5 if args.with_out else 1.0)

    # the read ceiling of the attention kernel's access pattern on this machine: its loads alone, (a) back to back
    # and (b) alternating with real decode steps' second half, as in the loop that was timed
    roco.roco_profile_kernel(roco.PROF_KERNELS["read_probe"])
    for _ in range(40):
        roco.roco_probe_cache_read(p, cache.K, cache.V, ws_d, stream=stream)
    torch.cuda.synchronize()
    ms, n = roco.roco_profile_read()
    probe_alone_s = ms * 1e-3 / max(1, n)
    # The same decode loop with the batch split into two halves (8 sequences each) on two HIP streams of default
    # priority: while one half's kernel is in its selection tail, or between two launches, the other half's streams.
    two_streams = None
    if (not args.no_two_streams and U % 2 == 0
            and roco.decode_step_launches(roco.RocoParams(U // 2, d, B, s, roco.ROCO_BF16)) == 1):
        Uh = U // 2
        ph = roco.RocoParams(Uh, d, B, s, roco.ROCO_BF16)
        phref = ctypes.byref(ph)
        ws_h = [torch.empty(roco.decode_workspace_bytes(ph), dtype=torch.uint8, device="cuda") for _ in range(2)]
        side = [torch.cuda.Stream(), torch.cuda.Stream()]
        rowh, cnth = Uh * d * esz, Uh * 4
        halves = []
        for h in range(2):
            halves.append((cK + h * Uh * B * d * esz, cV + h * Uh * B * d * esz, cS + h * Uh * 3 * B * 4,
                           cP + h * Uh * B * 4, cN + h * cnth, cX + h * cnth, ws_h[h].data_ptr(), ws_h[h].numel(),
                           side[h].cuda_stream))

        def decode_halves():
            for t in range(decode_steps):
                a = step_args[t]
                for h, (hK, hV, hS, hP, hN, hX, hw, hwb, hs) in enumerate(halves):
                    rc = lib.roco_decode_step(phref, a[0] + h * rowh, a[1] + h * rowh, a[2] + h * rowh, a[3] + h * cnth,
                                              hK, hV, hS, hP, hN, hX, a[4] + h * rowh, a[5] + h * cnth, a[6] + h * cnth,
                                              hw, hwb, hs)
                    if rc != 0:
                        raise roco.RocoError(rc, "roco_decode_step")

        for st in side:
            st.wait_stream(stream)
        decode_halves()  # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        decode_halves()
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t0
        stream.wait_stream(side[0]); stream.wait_stream(side[1])
        assert int(cache.n_used.min()) == B and int(cache.n_used.max()) == B
        two_streams = {"workload": "the same 16 sequences as two halves of 8 on two HIP streams, %d steps" % decode_steps,
                       "ms_per_token_step": dt2 / decode_steps * 1e3,
                       "tokens_per_s": cfg.batch * decode_steps / dt2,
                       "step_frac_of_hbm_peak": step_bytes / (dt2 / decode_steps) / 1e9 / HBM_PEAK_GBS}
    # a short extra pass (outside the timed region) with events around the two prefill statistics kernels
    pre_kernel_ms = {}
    for name in ("prefill_rows", "prefill_columns", "prefill_select", "prefill_gather"):
        roco.roco_profile_kernel(roco.PROF_KERNELS[name])
        for _ in range(5):  # back to back, as in the timed region
            prefill()
        torch.cuda.synchronize()
        ms, n = roco.roco_profile_read()
        pre_kernel_ms[name] = ms / max(1, n)
    roco.roco_profile_kernel(-1)
    # the same prefill when the caller also wants the prompt's attention output from pass 1 (1.5x the flops)
    with_output = None
    if not args.with_out:
        O2 = torch.empty_like(dQ)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for k in range(3):
            if k == 1:
                e0.record(stream)
            roco.roco_prefill_compress(p, dQ, dK, dV, dlen, L, cache.K, cache.V, cache.stats, cache.pos, cache.n_used,
                                       cache.next_slot, O2, ws_p, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 2
        tf = 1.5 * prefill_flops / (ms * 1e-3) / 1e12
        with_output = {"prefill_ms": ms, "prefill_evict_tokens_per_s": cfg.batch * L / (ms * 1e-3),
                       "achieved_TFLOPs": tf, "frac_of_mfma_peak": tf / MFMA_BF16_PEAK_TFLOPS}
        del O2
    # ... and when the caller's attention kernel already produced the row normalisers (pass 1 skipped).  The
    # normalisers are made here with torch as stand-ins for that kernel's output.
    given_lse = None
    if not args.with_out:
        lse = torch.empty((U, 1, L), dtype=torch.float32, device="cuda")
        causal = torch.ones((L, L), dtype=torch.bool, device="cuda").tril_()
        for i in range(0, U, 32):
            S = torch.matmul(dQ[i:i + 32].float(), dK[i:i + 32].float().transpose(1, 2)) * (1.0 / d ** 0.5)
            lse[i:i + 32, 0] = torch.logsumexp(S.masked_fill_(~causal, float("-inf")), dim=-1)
        del S, causal
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for k in range(6):
            if k == 1:
                e0.record(stream)
            roco.roco_prefill_compress_lse(p, 1, dQ, dK, dV, dlen, L, lse, cache.K, cache.V, cache.stats, cache.pos,
                                           cache.n_used, cache.next_slot, ws_p, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        given_lse = {"prefill_ms": ms, "prefill_evict_tokens_per_s": cfg.batch * L / (ms * 1e-3),
                     "achieved_TFLOPs": 0.5 * prefill_flops / (ms * 1e-3) / 1e12}
        assert int(cache.n_used.min()) == B and int(cache.n_used.max()) == B
        del lse
    dec_kernel_ms = {}
    for name in (() if fused else ("decode_finish",)):
        roco.roco_profile_kernel(roco.PROF_KERNELS[name])
        for t in range(min(32, decode_steps)):
            decode_one(t)
        torch.cuda.synchronize()
        ms, n = roco.roco_profile_read()
        dec_kernel_ms[name] = ms / max(1, n)
    # the matrix throughput this machine sustains (its clock under that load included): the prefill passes' matrix
    # instruction in a loop on register operands, and nothing else -- with operands of pseudo-random values (the bit
    # activity of real activations; the ceiling the prefill is compared with) and with a few constant small values
    roco.roco_profile_kernel(roco.PROF_KERNELS["mfma_probe"])
    sink = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
    mfma_ceiling = {}
    for random_operands in (True, False):
        probe_flops = 0
        for k in range(6):
            if k == 1:
                torch.cuda.synchronize()
                roco.roco_profile_read()  # the first launch is a warm-up
                probe_flops = 0
            probe_flops += roco.roco_probe_mfma(2048, 2048, sink, stream=stream, random_operands=random_operands)
        torch.cuda.synchronize()
        ms, n = roco.roco_profile_read()
        mfma_ceiling[random_operands] = probe_flops / (ms * 1e-3) / 1e12
    mfma_ceiling_tflops = mfma_ceiling[True]
    # ... and the ceiling of each pass's own instruction mix: the steady state of its pipelined form (matrix
    # instructions, fragment reads, the vector work per score) with no global loads, barriers or masks
    mix_ceiling = {}
    for which, mix in (("rows", 1), ("columns", 2)):
        probe_flops = 0
        for k in range(5):
            if k == 1:
                torch.cuda.synchronize()
                roco.roco_profile_read()
                probe_flops = 0
            probe_flops += roco.roco_probe_mfma(2048, 512, sink, stream=stream, mix=mix)
        torch.cuda.synchronize()
        ms, n = roco.roco_profile_read()
        mix_ceiling[which] = probe_flops / (ms * 1e-3) / 1e12
    # prefill repeated on its own: median and minimum of 10
    reps = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(10)]
    roco.roco_profile_kernel(-1)
    for e0, e1 in reps:
        e0.record(stream)
        prefill()
        e1.record(stream)
    torch.cuda.synchronize()
    rep_ms = sorted(e0.elapsed_time(e1) for e0, e1 in reps)
    dec_kernel_ms[attend_name] = attend_avg_s * 1e3
    dec_kernel_ms["read_probe"] = probe_alone_s * 1e3

    # Block-wise evict-and-encode (the paper's Table 6: speed-up of prompt encoding over token-wise eviction grows
    # like the block size): encode the same 512 tokens on the full cache in blocks of b, from the same start state.
    blockwise = None
    if not args.no_blockwise and decode_steps >= 32:
        n_tok = decode_steps - decode_steps % 32
        prefill()
        torch.cuda.synchronize()
        snap = [t.clone() for t in (cache.K, cache.V, cache.stats, cache.pos, cache.n_used, cache.next_slot)]
        bq, bk, bv = (x[:n_tok].transpose(0, 1).contiguous() for x in (sq, sk, sv))  # [U, n_tok, d]
        blockwise = {}
        for bsz in [int(x) for x in args.block_sizes.split(",") if x.strip()]:
            nb = n_tok // bsz
            tq, tk, tv = (x.view(U, nb, bsz, d).permute(1, 0, 2, 3).contiguous() for x in (bq, bk, bv))
            ws_b = torch.empty(roco.block_workspace_bytes(p, bsz), dtype=torch.uint8, device="cuda")
            bout = torch.empty((U, bsz, d), dtype=dt, device="cuda")
            qp0 = [torch.full((U,), L + i * bsz, dtype=torch.int32, device="cuda") for i in range(nb)]
            times = []
            for rep in range(2):
                for t, sn in zip((cache.K, cache.V, cache.stats, cache.pos, cache.n_used, cache.next_slot), snap):
                    t.copy_(sn)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for i in range(nb):
                    roco.roco_encode_block(p, bsz, tq[i], tk[i], tv[i], qp0[i], cache.K, cache.V, cache.stats, cache.pos,
                                           cache.n_used, cache.next_slot, bout, None, None, ws_b, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            ms = min(times)
            blockwise[str(bsz)] = {"tokens_per_s": cfg.batch * n_tok / (ms * 1e-3), "ms_per_block_step": ms / nb}
            del tq, tk, tv, ws_b
        if "1" in blockwise:
            for v in blockwise.values():
                v["speedup_vs_block_1"] = v["tokens_per_s"] / blockwise["1"]["tokens_per_s"]

        # The same table for the shapes the matrix cores do not take (workload 1's fp32 / head_dim 64), at workload 3's
        # bytes: 512 units x 2048 slots of fp32 / d=64 on a full cache with seeded Gaussian rows and valid statistics.
        blockwise_f32 = {}
        p32 = roco.RocoParams(U, 64, B, s, roco.ROCO_F32)
        c32 = roco.alloc_cache(p32)
        gen32 = torch.Generator(device="cuda").manual_seed(args.seed)
        for i0 in range(0, U, 64):
            c32.K[i0:i0 + 64] = torch.randn((min(64, U - i0), B, 64), device="cuda", generator=gen32)
            c32.V[i0:i0 + 64] = torch.randn((min(64, U - i0), B, 64), device="cuda", generator=gen32)
        cnt32 = torch.randint(1, 500, (U, B), device="cuda", generator=gen32).float()
        acc32 = torch.rand((U, B), device="cuda", generator=gen32) * cnt32 / B
        c32.stats[:, 0] = acc32
        c32.stats[:, 1] = acc32 * acc32 / cnt32 * (1 + torch.rand((U, B), device="cuda", generator=gen32))
        c32.stats[:, 2] = cnt32
        c32.n_used.fill_(B)
        c32.pos.copy_(torch.arange(B, device="cuda", dtype=torch.int32)[None].expand(U, B))
        ws_d32 = torch.empty(roco.decode_workspace_bytes(p32), dtype=torch.uint8, device="cuda")
        roco.roco_select_victims(p32, c32.stats, c32.pos, c32.n_used, c32.next_slot, ws_d32)
        torch.cuda.synchronize()
        snap32 = [t.clone() for t in (c32.stats, c32.pos, c32.n_used, c32.next_slot)]  # K / V rows only get overwritten
        n32 = 64
        for bsz in [b_ for b_ in (1, 8, 64) if str(b_) in blockwise]:
            nb = n32 // bsz
            tq = torch.randn((nb, U, bsz, 64), device="cuda", generator=gen32)
            tk = torch.randn((nb, U, bsz, 64), device="cuda", generator=gen32)
            tv = torch.randn((nb, U, bsz, 64), device="cuda", generator=gen32)
            ws_b = torch.empty(roco.block_workspace_bytes(p32, bsz), dtype=torch.uint8, device="cuda")
            bout = torch.empty((U, bsz, 64), dtype=torch.float32, device="cuda")
            qp0 = [torch.full((U,), B + i * bsz, dtype=torch.int32, device="cuda") for i in range(nb)]
            times = []
            for rep in range(2):
                for t, sn in zip((c32.stats, c32.pos, c32.n_used, c32.next_slot), snap32):
                    t.copy_(sn)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for i in range(nb):
                    roco.roco_encode_block(p32, bsz, tq[i], tk[i], tv[i], qp0[i], c32.K, c32.V, c32.stats, c32.pos,
                                           c32.n_used, c32.next_slot, bout, None, None, ws_b, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            ms = min(times)
            blockwise_f32[str(bsz)] = {"tokens_per_s": cfg.batch * n32 / (ms * 1e-3), "ms_per_block_step": ms / nb}
            del tq, tk, tv, ws_b
        if "1" in blockwise_f32:
            for v in blockwise_f32.values():
                v["speedup_vs_block_1"] = v["tokens_per_s"] / blockwise_f32["1"]["tokens_per_s"]
        del c32, snap32, ws_d32, cnt32, acc32

        # Grouped-query attention: the same 32 query heads per sequence over 32 / g key/value heads (g = 4 is the
        # Zephyr-style shape); one token per step.  The start state of each key/value head is a compressed cache.
        gqa = {}
        n_g = min(64, n_tok)
        for g in [int(x) for x in args.gqa_groups.split(",") if x.strip()]:
            Ug = U // g
            pg = roco.RocoParams(Ug, d, B, s, roco.ROCO_BF16)
            cg = roco.alloc_cache(pg)
            ws_g = torch.empty(roco.block_workspace_bytes(pg, 1), dtype=torch.uint8, device="cuda")
            gq = sq[:n_g].reshape(n_g, Ug, g, d).contiguous()
            gk, gv = sk[:n_g, :Ug].contiguous(), sv[:n_g, :Ug].contiguous()
            gout = torch.empty((Ug, g, d), dtype=dt, device="cuda")
            qps = [torch.full((Ug,), L + i, dtype=torch.int32, device="cuda") for i in range(n_g)]
            times = []
            for rep in range(2):
                for t, sn in zip((cg.K, cg.V, cg.stats, cg.pos, cg.n_used, cg.next_slot), snap):
                    t.copy_(sn[:Ug])
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for i in range(n_g):
                    roco.roco_decode_step_gqa(pg, g, gq[i], gk[i], gv[i], qps[i], cg.K, cg.V, cg.stats, cg.pos, cg.n_used,
                                              cg.next_slot, gout, None, None, ws_g, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            ms = min(times) / n_g
            # the grouped prompt: this workload's queries as g heads per key/value head, one-step eviction
            ws_pg = torch.empty(roco.prefill_gqa_workspace_bytes(pg, g, L), dtype=torch.uint8, device="cuda")
            gQ = dQ.view(Ug, g, L, d)
            glen = dlen[:Ug].contiguous()
            ptimes = []
            for rep in range(2):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                roco.roco_prefill_compress_gqa(pg, g, gQ, dK[:Ug], dV[:Ug], glen, L, cg.K, cg.V, cg.stats, cg.pos,
                                               cg.n_used, cg.next_slot, None, ws_pg, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                ptimes.append(e0.elapsed_time(e1))
            del ws_pg
            by_block = None
            if g == 4:  # appendix A's setting: a group of 4 encoded in blocks of up to 16 tokens (64 query rows)
                by_block = {}
                n_b = min(128, n_tok)
                for bsz in [int(x) for x in args.gqa_block_sizes.split(",") if x.strip()]:
                    nb = n_b // bsz
                    tq = sq[:n_b].reshape(nb, bsz, Ug, g, d).permute(0, 2, 1, 3, 4).contiguous()  # [nb, Ug, bsz, g, d]
                    tk = sk[:n_b, :Ug].reshape(nb, bsz, Ug, d).permute(0, 2, 1, 3).contiguous()
                    tv = sv[:n_b, :Ug].reshape(nb, bsz, Ug, d).permute(0, 2, 1, 3).contiguous()
                    ws_gb = torch.empty(roco.block_workspace_bytes(pg, bsz), dtype=torch.uint8, device="cuda")
                    gbout = torch.empty((Ug, bsz, g, d), dtype=dt, device="cuda")
                    qp0 = [torch.full((Ug,), L + i * bsz, dtype=torch.int32, device="cuda") for i in range(nb)]
                    btimes = []
                    for rep in range(2):
                        for t, sn in zip((cg.K, cg.V, cg.stats, cg.pos, cg.n_used, cg.next_slot), snap):
                            t.copy_(sn[:Ug])
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record(stream)
                        for i in range(nb):
                            roco.roco_encode_block_gqa(pg, bsz, g, tq[i], tk[i], tv[i], qp0[i], cg.K, cg.V, cg.stats, cg.pos,
                                                       cg.n_used, cg.next_slot, gbout, None, None, ws_gb, stream=stream)
                        e1.record(stream)
                        torch.cuda.synchronize()
                        btimes.append(e0.elapsed_time(e1))
                    bms = min(btimes)
                    by_block[str(bsz)] = {"tokens_per_s": cfg.batch * n_b / (bms * 1e-3), "ms_per_block_step": bms / nb}
                    del tq, tk, tv, ws_gb, gbout
                if "1" in by_block:
                    for v in by_block.values():
                        v["speedup_vs_block_1"] = v["tokens_per_s"] / by_block["1"]["tokens_per_s"]
            gqa[str(g)] = {"kv_heads_per_layer": 32 // g, "units": Ug, "ms_per_token_step": ms,
                           "encode_by_block_size": by_block,
                           "prefill_evict_ms": min(ptimes), "prefill_evict_tokens_per_s": cfg.batch * L / (min(ptimes) * 1e-3),
                           "tokens_per_s": cfg.batch / (ms * 1e-3),
                           "cache_read_GBps": Ug * B * d * 2 * 2 / (ms * 1e-3) / 1e9}
            del cg, ws_g, gq, gk, gv
        del snap

    result = {
        "metric": "RoCo decode tokens/s (7B-shape layer, B=2048, batch 16); prefill+evict tok/s",
        "value": decode_tok_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "config 3: 7B-shaped layer, 32 heads x 128 dims bf16, batch 16, prompt 3072 -> B=2048, "
                               f"scope 64, {decode_steps} decode steps", "units": U, "budget": B, "scope": s,
                   "prompt_len": L, "decode_steps": decode_steps, "batch": cfg.batch, "seed": args.seed,
                   "prefill_attention_output": bool(args.with_out)},
        "decode_ms_per_token_step": decode_ms / (decode_steps * args.steps),
        "prefill_evict_tokens_per_s": prefill_tok_s,
        "prefill_ms": prefill_ms / args.steps,
        "roofline": {"kernel": attend_name, "bound": "hbm", "achieved": attend_bytes / attend_avg_s / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": attend_bytes / attend_avg_s / 1e9 / HBM_PEAK_GBS,
                     "traffic": (traffic or {}).get("bytes"), "traffic_source": traffic,
                     "bytes_per_launch": attend_bytes, "avg_launch_ms": attend_avg_s * 1e3, "launches": attend_n,
                     "measured_read_ceiling_GBps": U * B * 2 * d * esz / probe_alone_s / 1e9,
                     "frac_of_measured_ceiling": attend_bytes / attend_avg_s / (U * B * 2 * d * esz / probe_alone_s)},
        "roofline_decode_step": {"bound": "hbm", "achieved": step_bytes / (decode_ms * 1e-3 / (decode_steps * args.steps)) / 1e9,
                                 "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": step_bytes / (decode_ms * 1e-3 / (decode_steps * args.steps)) / 1e9 / HBM_PEAK_GBS,
                                 "bytes_per_step": step_bytes},
        "decode_two_streams": two_streams,
        "prefill_with_attention_output": with_output,
        "prefill_given_row_normalisers": given_lse,
        "roofline_prefill": {"bound": "mfma", "achieved": prefill_flops / (prefill_ms * 1e-3 / args.steps) / 1e12,
                             "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": prefill_flops / (prefill_ms * 1e-3 / args.steps) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                             "flops_per_pass": prefill_flops,
                             "measured_mfma_ceiling_TFLOPs": mfma_ceiling_tflops,
                             "measured_mfma_ceiling_constant_operands_TFLOPs": mfma_ceiling[False],
                             "frac_of_measured_ceiling": prefill_flops / (prefill_ms * 1e-3 / args.steps) / 1e12
                             / mfma_ceiling_tflops,
                             "prefill_ms_median_of_10": rep_ms[len(rep_ms) // 2], "prefill_ms_min_of_10": rep_ms[0]},
        "roofline_prefill_kernels": {
            which: {"kernel": kname, "bound": "alu", "avg_launch_ms": pre_kernel_ms[key],
                    "achieved": prefill_flops / 2 / (pre_kernel_ms[key] * 1e-3) / 1e12, "unit": "TFLOP/s",
                    "peak": alu_cobound_tflops(which),
                    "frac": prefill_flops / 2 / (pre_kernel_ms[key] * 1e-3) / 1e12 / alu_cobound_tflops(which),
                    "frac_of_mfma_peak": prefill_flops / 2 / (pre_kernel_ms[key] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                    "measured_mix_ceiling_TFLOPs": mix_ceiling[which],
                    "frac_of_measured_mix_ceiling": prefill_flops / 2 / (pre_kernel_ms[key] * 1e-3) / 1e12 / mix_ceiling[which],
                    "issue_bound_at_counted_mix": counted_issue_bound_tflops(kname, 3) if U == 512 else None,
                    "traffic": (measured_traffic(kname, 3) or {}).get("bytes") if U == 512 else None,
                    "traffic_source": measured_traffic(kname, 3) if U == 512 else None,
                    "algorithmic_bytes": 2 * U * L * d * esz}
            for which, kname, key in (("rows", "prefill_rows_mfma", "prefill_rows"), ("columns", "prefill_columns_mfma", "prefill_columns"))
        } if not args.with_out else None,
        "kernel_ms": {**dec_kernel_ms, **pre_kernel_ms},
        "input_generation_s": t_gen,
    }
    if blockwise is not None:
        result["blockwise_encode"] = {"workload": f"{n_tok} tokens per sequence encoded on the full B={B} cache in "
                                                  "blocks of b (roco_encode_block), batch 16 x 32 heads",
                                      "by_block_size": blockwise,
                                      "fp32_head_dim_64": {
                                          "workload": f"64 tokens per sequence in blocks of b on a full B={B} cache of fp32 / "
                                                      "head_dim 64 rows (vector-ALU kernel), same units and bytes",
                                          "by_block_size": blockwise_f32}}
        result["gqa"] = {"workload": f"32 query heads over 32/g key/value heads, batch 16: the {L}-token prompt compressed "
                                     f"to B={B} (roco_prefill_compress_gqa), then one token per step on the full "
                                     "cache (roco_decode_step_gqa)", "by_group_size": gqa}
    if not args.no_consistency:
        # section 4.1's consistency study on this workload's generator (32 heads of sequence 0, 256-token prompt,
        # 256 generated tokens): Jaccard similarity between what a budgeted cache holds and the top-B tokens of
        # the same importance score with the full cache, scope = whole cache
        from inputs import make_unit, unit_ids
        from paper_2402_06262_amd.consistency import consistency_study
        ids = unit_ids(cfg)[:32]
        small = [make_unit(cfg, *i, seed=args.seed, total_len=512) for i in ids]
        cq, ck, cv = (upload(np.stack([getattr(u_, n_) for u_ in small]), torch, dt) for n_ in ("Q", "K", "V"))
        t0c = time.perf_counter()
        study = consistency_study(cq, ck, cv, prompt_len=256, rates=(0.3, 0.4, 0.5, 0.6), importances=("mas", "aas", "aqas", "ltas"))
        result["consistency_synthetic"] = {
            "workload": "32 units of this workload's generator, 256-token prompt + 256 generated tokens, budget = "
                        "rate x 512, scope = whole cache, every 8th position",
            "jaccard_vs_full_cache": {k_: {str(r_): round(v_[0], 4) for r_, v_ in d_.items()} for k_, d_ in study.items()},
            "seconds": round(time.perf_counter() - t0c, 2)}
        del cq, ck, cv
    which = [int(x) for x in args.workloads.split(",") if x.strip()]
    if which:
        del dQ, dK, dV, sq, sk, sv, out, cache
        torch.cuda.empty_cache()
        result["workloads"] = side_workloads(torch, roco, args.seed, which)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, Q, K, V, decode_steps, args.cpu_units, args.cpu_steps)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
