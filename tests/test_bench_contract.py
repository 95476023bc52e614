"""CPU checks of bench.py's host side: what it reads from profiles/, the bounds it prices the prefill passes against,
and that it refuses more than one GPU (nothing here touches a GPU)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_counted_traffic_is_read_per_kernel_and_workload_and_never_carried_over():
    for kernel in ("decode_fused", "prefill_rows_mfma", "prefill_columns_mfma", "prefill_gather", "prefill_select"):
        t = bench.measured_traffic(kernel, 3)
        assert t is not None, kernel
        assert t["bytes"] == t["fetch_bytes"] + t["write_bytes"] > 0
        assert t["kernel"] == kernel and len(t["measured_at_commit"]) >= 7 and t["source"].startswith("profiles/")
    # the decode step of workload 3 moves its 562 MB once: the counted bytes are within 2 % of the algorithmic ones
    alg = 2048 * (2 * 128 * 2 + 24) * 512
    assert abs(bench.measured_traffic("decode_fused", 3)["bytes"] / alg - 1.0) < 0.02
    assert bench.measured_traffic("decode_fused", 4) is None  # another workload: no figure
    assert bench.measured_traffic("no_such_kernel", 3) is None


def test_issue_bounds_follow_from_the_slot_counts():
    # 9 / 11 issue slots of 4 cycles against the matrix instruction's 32 cycles (two scores per lane per instruction:
    # multiply-add, exponential (two slots), add -- and one more multiply-add in the column pass -- plus its own slot)
    assert bench.alu_cobound_tflops("rows") == pytest.approx(bench.MFMA_BF16_PEAK_TFLOPS * 32 / 36)
    assert bench.alu_cobound_tflops("columns") == pytest.approx(bench.MFMA_BF16_PEAK_TFLOPS * 32 / 44)
    for kernel, ideal in (("prefill_rows_mfma", 9.0), ("prefill_columns_mfma", 11.0)):
        c = bench.counted_issue_bound_tflops(kernel, 3)
        assert c is not None
        assert c["issue_slots_per_mfma"] >= ideal  # the kernels cannot issue fewer than the arithmetic needs
        assert c["TFLOPs"] == pytest.approx(bench.MFMA_BF16_PEAK_TFLOPS * 32 / (4 * c["issue_slots_per_mfma"]))
    assert bench.counted_issue_bound_tflops("prefill_rows_mfma", 5) is None


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=300)
    assert run.returncode != 0
    assert "--gpus 1" in run.stderr and run.stdout.strip() == ""
