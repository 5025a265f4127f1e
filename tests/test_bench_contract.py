"""bench.py's command-line contract: more than one GPU is refused with a message
(CPU), and the default single-GPU run prints one JSON line with the agreed keys
(GPU)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_single_gpu_run_prints_one_json_line_with_the_agreed_keys():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "20",
                        "--warmup", "5", "--no-points"], capture_output=True, text=True,
                       timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    rec = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config",
                "roofline", "cpu_baseline"):
        assert key in rec, key
    assert rec["n_gpus"] == 1 and rec["steps"] == 20 and rec["warmup"] == 5
    assert rec["vs_baseline"] is None and rec["data"] == "synthetic" and rec["dtype"] == "bf16"
    assert "workload" in rec["config"] and "model" not in rec["config"]
    roof = rec["roofline"]
    assert roof["bound"] in ("hbm", "mfma") and roof["unit"] in ("GB/s", "TFLOP/s")
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert 0.3 < roof["frac"] < 1.0                  # an HBM-bound kernel cannot beat the peak
    # measured HBM bytes per launch, carried from the tracked counter summary while the
    # kernel sources are what they were then; a streaming kernel reads its weights once
    assert roof["traffic"] is None or 0.95 < roof["traffic_over_algorithmic"] < 1.2
    cpu = rec["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    assert rec["value"] > 10 * cpu["value"]
    assert abs(rec["value"] - 64 / (rec["ms_per_step"] * 1e-3)) < 1e-6 * rec["value"]


def test_traffic_table_is_used_only_while_the_kernel_sources_are_unchanged(monkeypatch):
    """roofline.traffic comes from profiles/traffic.json (counter runs summarised by
    paper_2605_14438_amd.profile_summary); a record is dropped as soon as the kernel's source
    files no longer hash to what they were when it was taken."""
    sys.path.insert(0, ROOT)
    import bench
    table = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    recs = table["records"]
    assert recs, "the traffic table is empty"
    for r in recs:
        assert r["kernel"] in ("gate_up", "down")
        assert r["fetch_bytes"] > 0 and r["write_bytes"] >= 0 and r["forwards"] > 0
        assert r["profile"].startswith("profiles/") and os.path.exists(os.path.join(ROOT, r["profile"]))
        for f in r["source_files"]:
            assert os.path.exists(os.path.join(ROOT, f)), f
        got = bench.measured_traffic(r["workload"], r["kernel"])
        if bench._sha16(r["source_files"]) == r["source_sha16"]:
            assert got["bytes"] == r["fetch_bytes"] + r["write_bytes"]
        else:
            assert got is None
    r = recs[0]
    monkeypatch.setattr(bench, "_sha16", lambda paths: "0" * 16)
    assert bench.measured_traffic(r["workload"], r["kernel"]) is None
    assert bench.measured_traffic("no such workload", "gate_up") is None
