"""bench.py's command-line contract: one GPU only, ONE JSON line with the agreed keys."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figures_come_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.parse_traffic()
    assert t, "profiles/lsp_step_hbm_traffic_counters.txt has no sections"
    c4 = bench.traffic_for("c4", "lsp_attn_step", 32)
    # K/V + Q read once and O written once per layer: 805 MB (cache 2 x 8 x 5120 rows x 8 KB, Q and O 67 MB each)
    assert c4 is not None and 0.98 < c4 / (32 * 805.3e6) < 1.05
    assert bench.traffic_for("c2", "lsp_confidence", 1) is not None
    assert bench.traffic_for("no_such_workload", "lsp_confidence", 1) is None


@pytest.mark.gpu
def test_one_json_line_with_roofline_and_cpu_baseline_on_the_tiny_configuration():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "c1", "--steps", "4", "--warmup", "2", "--also", ""],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 4 and d["warmup"] == 2 and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["config"]["workload"].startswith("c1") and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] in ("hbm", "mfma", "alu") and rf["achieved"] > 0 and rf["peak"] > 0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
