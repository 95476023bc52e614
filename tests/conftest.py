import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, on a machine without a GPU (plain `pytest tests/`).
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """After a GPU run: the declared ties of every workload that counted them, and how far the attention outputs were
    from the oracle in units of their tolerance (shown whatever the verbosity)."""
    parity = sys.modules.get("parity")
    if parity is None or not (parity.TIE_LOG or any(w[0] for w in parity.WORST_OUT.values())):
        return
    tr = terminalreporter
    tr.write_line("declared ties (decisions where library and oracle differ inside the tolerance band):")
    pd = pt = dd = dt = 0
    for what, a, b, c, d in parity.TIE_LOG:
        pd, pt, dd, dt = pd + a, pt + b, dd + c, dt + d
        if b or d:
            tr.write_line(f"  {what}: prefill {b}/{a}, decode {d}/{c}")
    tr.write_line(f"  total: prefill {pt}/{pd}, decode {dt}/{dd} over {len(parity.TIE_LOG)} workloads")
    for dtype, (used, strict) in parity.WORST_OUT.items():
        tr.write_line(f"worst attention-output error, {dtype}: {used:.3f} of the tolerance with the floor rms(o); "
                      f"{strict:.3f} with the floor 1e-3 * rms(o)")
    tr.write_line(f"worst Acc / Acc2 error: {parity.WORST_STAT[0]:.3g} relative (tolerance {parity.STAT_RTOL:g}, "
                  f"floor {parity.STAT_FLOOR:g})")
