"""The benchmark aids of the library run and leave the state they are given alone: the matrix-instruction probes in
their four modes, the loads-only probe of the decode step, and the per-kernel event timing."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["constant", "random", "row-mix", "column-mix"])
def test_matrix_probe_runs_in_every_mode_and_fills_its_sink(mode):
    import paper_2402_06262_amd as roco
    workgroups, iters = 16, 8
    sink = torch.full((workgroups * 256,), float("nan"), dtype=torch.float32, device="cuda")
    kw = {"constant": {}, "random": dict(random_operands=True), "row-mix": dict(mix=1), "column-mix": dict(mix=2)}[mode]
    flops = roco.roco_probe_mfma(workgroups, iters, sink, **kw)
    torch.cuda.synchronize()
    assert flops == workgroups * 4 * iters * (32 if "mix" in mode else 8) * 32768
    assert torch.isfinite(sink).all()  # every thread wrote its checksum
    with pytest.raises(roco.RocoError):  # a sink too small for the grid is refused on the host
        roco.roco_probe_mfma(workgroups, iters, sink[:-1], **kw)


def test_cache_read_probe_and_kernel_timing_leave_the_cache_alone():
    import paper_2402_06262_amd as roco
    units, d, B, s = 130, 128, 512, 16
    p = roco.RocoParams(units, d, B, s, roco.ROCO_BF16)
    c = roco.alloc_cache(p)
    torch.manual_seed(1)
    c.K.copy_(torch.randn(units, B, d, device="cuda").to(torch.bfloat16))
    c.V.copy_(torch.randn(units, B, d, device="cuda").to(torch.bfloat16))
    before = (c.K.clone(), c.V.clone())
    ws = torch.empty(max(16, roco.decode_workspace_bytes(p)), dtype=torch.uint8, device="cuda")
    roco.roco_profile_read()
    roco.roco_profile_kernel(roco.PROF_KERNELS["read_probe"])
    for _ in range(3):
        roco.roco_probe_cache_read(p, c.K, c.V, ws)
    torch.cuda.synchronize()
    ms, n = roco.roco_profile_read()
    roco.roco_profile_kernel(-1)
    assert n == 3 and 0.0 < ms < 100.0
    assert torch.equal(before[0], c.K) and torch.equal(before[1], c.V)
