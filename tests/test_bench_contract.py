"""Host-side contract of bench.py: one GPU only, and the result line carries the agreed keys."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_world_size_above_one_is_refused():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, cwd=ROOT, env=env)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)


@pytest.mark.gpu
def test_result_line_has_the_contract_keys():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "1", "--steps", "2", "--warmup", "1",
                        "--cpu-tokens", "64"], capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    res = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in res, k
    assert res["n_gpus"] == 1 and res["steps"] == 2 and res["warmup"] == 1 and res["vs_baseline"] is None
    assert "workload" in res["config"] and res["data"] == "synthetic"
    rf = res["roofline"]
    assert set(("bound", "achieved", "peak", "unit", "frac", "traffic")) <= set(rf)
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    assert {"measured_peak", "frac_of_measured", "per_group", "median_ms_per_step", "min_ms_per_step"} <= set(rf)
    assert rf["measured_peak"]["mfma_TFLOP/s"] > 100 and rf["measured_peak"]["copy_GB/s"] > 500
    gate = res["per_call"]["gate_topk"]
    assert {"ms", "median_ms", "min_ms", "hbm_frac", "matrix_frac", "bound"} <= set(gate)
    cb = res["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]


def test_traffic_comes_from_the_counter_summary_and_names_its_workload():
    """roofline.traffic is parsed from the committed counter summary; a summary of another workload is refused."""
    sys.path.insert(0, ROOT)
    import bench
    path = bench.TRAFFIC_PROFILES[3]
    text = open(path).read()
    import re
    flops = float(re.search(r"algorithmic flops per step ([0-9.eE+]+)", text).group(1))
    t = bench.measured_traffic(3, flops)
    assert t is not None and 1e10 < t < 1e12
    assert bench.measured_traffic(1, 1.0) is None                    # no summary for that configuration
    with pytest.raises(SystemExit):
        bench.measured_traffic(3, flops * 1.1)


def test_group_bounds_follow_the_rooflines():
    """A group of few rows is bound by its weight bytes, a large one by the matrix cores; an empty one still pays
    for writing its gradients."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2411_10003_amd import workload as wl
    cfg = wl.CONFIGS[4]
    gb = bench.ffn_group_bounds(cfg, [0, 40, 12000], True)
    assert [g["bound"] for g in gb] == ["hbm", "hbm", "mfma"]
    assert abs(gb[0]["bound_us"] - (2 * cfg.d * cfg.h * 4) / 8e12 * 1e6) < 0.1      # an empty group: only its zero gradients
    assert abs(gb[2]["bound_us"] - 3 * 2.0 * 12000 * cfg.d * cfg.h * 2 / 2.5e15 * 1e6) < 0.1
