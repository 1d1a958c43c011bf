"""Host-only checks of bench.py: the one-GPU rule, the traffic record and the workload table."""
import json
import os
import subprocess
import sys

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_traffic_record_is_used_only_for_the_sources_it_was_measured_on(monkeypatch):
    with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
        rec = json.load(f)["resnet50_i8_stream"]
    assert rec["sources"] == list(bench.CONV_SOURCES)
    assert rec["hbm_bytes_per_launch"] == rec["read"] + rec["written"] > 0
    got = bench.measured_traffic("resnet50_i8_stream")
    assert got == (rec["hbm_bytes_per_launch"] if rec["kernel_sha256"] == bench.conv_sources_digest() else None)
    assert bench.measured_traffic("no_such_workload") is None
    monkeypatch.setattr(bench, "conv_sources_digest", lambda: "0" * 64)          # the kernel has changed: no figure
    assert bench.measured_traffic("resnet50_i8_stream") is None


def test_every_workload_names_a_calibrated_network():
    for name, wl in bench.WORKLOADS.items():
        assert wl["net"] in W.CONFIGS, name
        assert os.path.exists(os.path.join(ROOT, "workloads", "calib", wl["net"] + ".json")), name
        assert 1 <= wl["b_max"] <= 1024 and wl["refill"] in (0, 1, 2) and wl["n"] >= wl["b_max"]
