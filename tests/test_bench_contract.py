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


def test_recorded_traffic_is_reported_only_for_the_kernel_source_it_was_measured_on(tmp_path, monkeypatch):
    import hashlib

    src, sched = tmp_path / "ffn.hip", tmp_path / "schedule.h"
    src.write_text("kernel v1")
    sched.write_text("schedule v1")
    sha = hashlib.sha1(b"kernel v1schedule v1").hexdigest()[:12]
    table = tmp_path / "traffic.md"
    table.write_text("| workload | mode | scope | gamma | kernel | read bytes | written bytes | source |\n|---|---|---|---|---|---|---|---|\n"
                     f"| mixtral | token | local | 1 | ffn_gate_up | 5.0e9 | 2.5e8 | {sha} |\n"
                     f"| mixtral | token | local | 1 | ffn_down | 2.0e9 | 7.0e7 | 000000000000 |\n")
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(table))
    monkeypatch.setattr(bench, "KERNEL_SOURCES", [str(src), str(sched)])
    assert bench.recorded_traffic("mixtral", "token", "local", 1.0, "ffn_gate_up") == pytest.approx(5.25e9)
    assert bench.recorded_traffic("mixtral", "token", "local", 1.0, "ffn_down") is None      # another source version
    assert bench.recorded_traffic("mixtral", "expanded", "local", 1.0, "ffn_gate_up") is None
    sched.write_text("schedule v2")                                                           # the schedule changed
    assert bench.recorded_traffic("mixtral", "token", "local", 1.0, "ffn_gate_up") is None
    sched.write_text("schedule v1")
    assert bench.recorded_traffic("mixtral", "token", "local", 1.0, "ffn_gate_up") == pytest.approx(5.25e9)
    src.write_text("kernel v2")                                                               # the kernel changed
    assert bench.recorded_traffic("mixtral", "token", "local", 1.0, "ffn_gate_up") is None
    # the tracked table parses, whatever it holds today
    monkeypatch.undo()
    v = bench.recorded_traffic("mixtral", "token", "local", 1.0, "ffn_gate_up")
    assert v is None or v > 1e9


def test_defaults_name_the_headline_workload():
    old = sys.argv
    sys.argv = ["bench.py"]
    try:
        a = bench.parse()
    finally:
        sys.argv = old
    # the largest single-GPU configuration (the Mixtral-shaped layer), Token Drop with the Expanded Drop line beside it
    assert (a.gpus, a.workload, a.mode, a.scope, a.gamma, a.metric) == (1, "mixtral", "token", "local", 1.0, "score")
    assert not a.no_expanded and a.steps >= 50 and a.warmup >= 10
    assert [float(g) for g in a.sweep_gamma.split(",")][:4] == [0.5, 1.0, 1.5, 2.0]
