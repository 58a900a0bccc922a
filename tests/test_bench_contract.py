"""Host-side checks of bench.py: the roofline arithmetic and the command-line contract (no GPU needed)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402

from paper_2503_05066_amd import synth  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_binding_roof_is_the_slower_one():
    # 1 GFLOP and 1 GB: at 2.5 PFLOP/s and 8 TB/s the bytes take longer
    first, second = bench.roofline_of({"flops": 1e9, "bytes": 1e9}, ms=1.0)
    assert first["bound"] == "hbm" and second["bound"] == "mfma"
    assert first["achieved"] == pytest.approx(1e9 / 1e-3 / 1e9) and first["peak"] == 8000.0
    assert first["frac"] == pytest.approx(first["achieved"] / first["peak"])
    # 1 PFLOP of work on 1 MB: the matrix cores bind
    first, _ = bench.roofline_of({"flops": 1e15, "bytes": 1e6}, ms=1000.0)
    assert first["bound"] == "mfma" and first["unit"] == "TFLOP/s" and first["frac"] == pytest.approx(1000.0 / 2500.0)


def test_algorithmic_work_matches_the_stated_formulas():
    w = synth.WORKLOADS["olmoe"]
    rows, active, elem = 13701, 64, 2
    work = bench.algorithmic_work(w, w.top_k, rows, active, elem)
    n, d, e, k, h = w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden
    assert work["ffn_gate_up"]["bytes"] == active * 2 * h * d * elem + rows * (d + h) * elem
    assert work["ffn_gate_up"]["flops"] == 4 * d * h * rows and work["ffn_down"]["flops"] == 2 * d * h * rows
    assert work["combine"]["bytes"] == rows * d * elem + n * d * elem
    assert work["router_logits"]["bytes"] == n * d * elem + e * d * 4 + n * e * 4
    # the constant quoted for the measured traffic belongs to the default workload only
    assert list(bench.MEASURED_TRAFFIC) == [("olmoe", "token", "local", 1.0)]
    assert 0.9 < bench.MEASURED_TRAFFIC[("olmoe", "token", "local", 1.0)] / work["ffn_gate_up"]["bytes"] < 1.5


def test_defaults_name_the_headline_workload():
    old = sys.argv
    sys.argv = ["bench.py"]
    try:
        a = bench.parse()
    finally:
        sys.argv = old
    assert (a.gpus, a.workload, a.mode, a.scope, a.gamma, a.metric) == (1, "olmoe", "token", "local", 1.0, "score")
    assert a.steps >= 50 and a.warmup >= 10
