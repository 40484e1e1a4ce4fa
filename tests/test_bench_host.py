"""The parts of bench.py that need no GPU: the refusal of more than one GPU, and the check that the
counter traffic it reports belongs to the kernels it measures."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench                                               # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_counter_traffic_is_refused_when_the_kernels_changed(tmp_path, monkeypatch):
    f = tmp_path / "traffic.json"
    f.write_text(json.dumps({"cfg5": {"gap": {"kernels": ["gap_dense_kernel"], "bytes_per_launch": 1.5e9},
                                      "cd_pass": {"kernels": ["old_kernel"], "bytes_per_pass": 2.5e8}}}))
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    assert bench.counter_traffic("cfg5", "gap", ["gap_dense_kernel"]) == 1.5e9
    assert bench.counter_traffic("cfg2", "gap", ["gap_dense_kernel"]) is None          # not profiled: no figure
    with pytest.raises(SystemExit):
        bench.counter_traffic("cfg5", "cd_pass", ["cd_dense_worker_kernel", "merge_workers_kernel"])
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "missing.json"))
    assert bench.counter_traffic("cfg5", "gap", ["gap_dense_kernel"]) is None


def test_the_tracked_traffic_file_names_the_kernels_bench_measures():
    data = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    dense = {"cols": None, "d": 50000, "n": 500000, "m": 50000, "host_resident": False}
    sparse = {"val": None}
    for name, entry in data.items():
        gap, cd = bench.dominant_kernels(sparse if name == "cfg3" else dense, "async")
        assert entry["gap"]["kernels"] == gap and entry["cd_pass"]["kernels"] == cd, name
        assert entry["gap"]["bytes_per_launch"] > 0 and entry["cd_pass"]["bytes_per_pass"] > 0
