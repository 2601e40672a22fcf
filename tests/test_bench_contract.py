"""bench.py's command-line contract: one GPU only, one JSON line with the roofline and CPU-baseline objects."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_loop_policies_use_the_settings_the_paper_states():
    """Section 3: limit 40, Constant 5, Heuristic +2 / -1, T = 1, h = 0.3 (fixture with the citation)."""
    sys.path.insert(0, ROOT)
    import bench
    vals = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_hyperparameters.txt")):
        if line.strip() and not line.startswith("#"):
            key, *rest = line.split()
            vals[key] = [float(x) for x in rest]
    for key, v in bench.PAPER.items():
        assert vals[key] == [float(v)], key
    assert vals["entropy_threshold_grid"] == [0.2, 0.3, 0.4, 0.5] and bench.PAPER["entropy_threshold_h"] in vals["entropy_threshold_grid"]


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_required_objects():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "4", "--warmup", "2",
                        "--cpu-seqs", "2"], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "roofline_calls", "kernels", "stream_read_peak",
                "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 4 and d["warmup"] == 2 and d["unit"] == "rows/s"
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and "workload" in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and 0.05 < r["frac"] < 1.0
    # the roofline object describes the kernel that holds the largest share of the step
    ks = d["kernels"]
    assert set(ks) == {"k_draft_stats", "k_draft_finish", "k_verify_stats", "k_accept", "k_resid"}
    top = max(ks, key=lambda n: ks[n]["us_per_step"])
    assert r["kernel"].startswith(top) and r["bytes_per_launch"] == ks[top]["bytes_per_launch"]
    assert abs(sum(k["share_of_step_kernel_time"] for k in ks.values()) - 1.0) < 1e-9
    assert ks["k_verify_stats"]["bytes_per_launch"] == 64 * 17 * 128256 * 2
    assert ks["k_draft_stats"]["bytes_per_launch"] == 64 * 128256 * 2 and ks["k_draft_stats"]["launches_per_step"] == 16
    # the calls, priced on algorithmic bytes: nothing beats the peak, the step is the sum of its parts
    rc = d["roofline_calls"]
    for name in ("draft_step", "verify", "whole_step"):
        assert 0 < rc[name]["frac"] < 1.0 and abs(rc[name]["frac"] - rc[name]["GBps"] / 8000.0) < 1e-9
    assert rc["whole_step"]["bytes"] == 16 * rc["draft_step"]["bytes"] + rc["verify"]["bytes"]
    assert abs(rc["whole_step"]["us"] - 1e3 * d["ms_per_step"]) < 1e-6
    sum_kernels = sum(k["us_per_step"] for k in ks.values())
    # Kernel time against the wall time of the step: the kernels are timed one by one in eager launches, the
    # step is a graph replay in which a kernel starts while its predecessor's last waves drain, so the sum of
    # the durations comes out 5-13 % above the step (the rocprofv3 trace under profiles/ shows the same); the
    # bound only catches a sum that cannot belong to this step.
    assert sum_kernels < 1.25 * rc["whole_step"]["us"]
    sp = d["stream_read_peak"]
    assert 0.5 < sp["frac_of_hbm_peak"] < 1.0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "rows/s" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
    assert c["one_thread_rows_per_s"] > 0 and c["os_cpu_count"] >= 1
    assert d["value"] > 100 * c["value"]
