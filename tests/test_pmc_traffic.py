"""pmc_traffic.py turns two rocprofv3 counter runs into the file bench.py reads its `traffic` from: the
arithmetic of that step, on small made-up counter files (CPU only)."""
import csv
import json
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import pmc_traffic                                         # noqa: E402


def _write(path, counter, rows):
    os.makedirs(path, exist_ok=True)
    with open(os.path.join(path, "x_counter_collection.csv"), "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=["Kernel_Name", "Counter_Name", "Counter_Value"])
        w.writeheader()
        for name, value in rows:
            w.writerow({"Kernel_Name": name, "Counter_Name": counter, "Counter_Value": value})


def test_traffic_from_made_up_counters(tmp_path, monkeypatch):
    gib4_kib = 4.0 * (1 << 20)
    gap = "void duhl::(anonymous namespace)::gap_dense_kernel<0, 4, true, false>(duhl::GapArgs)"
    gap_norms = "void duhl::(anonymous namespace)::gap_dense_kernel<0, 4, true, true>(duhl::GapArgs)"
    worker = "void duhl::(anonymous namespace)::cd_dense_worker_kernel<0, 1024, 8, 5, true, false, true, 1>(duhl::CdArgs, long)"
    merge = "void duhl::(anonymous namespace)::merge_workers_kernel<64>(float*, long)"
    select = "void duhl::(anonymous namespace)::select_fused_kernel<16>(duhl::SelectArgs)"
    copy = "__amd_rocclr_copyBuffer"
    # FETCH_SIZE counts 2 KiB per unit here, WRITE_SIZE 1 KiB: the 4 GiB copy calibrates both
    _write(tmp_path / "f", "FETCH_SIZE", [(copy, gib4_kib / 2), (copy, 10.0), (gap, 1000.0), (gap, 1200.0),
                                           (gap_norms, 9e9), (worker, 300.0), (worker, 300.0), (worker, 300.0),
                                           (worker, 300.0), (merge, 10.0), (merge, 10.0), (merge, 10.0), (merge, 10.0),
                                           (select, 1.0), (select, 1.0)])
    _write(tmp_path / "w", "WRITE_SIZE", [(copy, gib4_kib), (gap, 8.0), (gap, 8.0), (gap_norms, 9e9),
                                           (worker, 40.0)] * 1 + [(worker, 40.0)] * 3 + [(merge, 4.0)] * 4
                                          + [(select, 1.0), (select, 1.0)])
    out = tmp_path / "traffic.json"
    monkeypatch.setattr(pmc_traffic, "TRAFFIC", str(out))
    monkeypatch.setattr(sys, "argv", ["pmc_traffic.py", "--workload", "toy", "--fetch", str(tmp_path / "f"),
                                      "--write", str(tmp_path / "w")])
    pmc_traffic.main()
    got = json.load(open(out))["toy"]
    assert got["calibration"]["FETCH_SIZE_KiB_per_count"] == pytest.approx(2.0)
    assert got["calibration"]["WRITE_SIZE_KiB_per_count"] == pytest.approx(1.0)
    # the gap launch: mean of the two dispatches (the instance that also computes the norms is set_data's)
    assert got["gap"]["bytes_per_launch"] == pytest.approx((1100.0 * 2.0 + 8.0 * 1.0) * 1024.0)
    assert got["gap"]["kernels"] == ["gap_dense_kernel"]
    # a pass: two selections = two rounds; four dispatches of each kernel = two per pass
    per_pass = 2 * (300.0 * 2.0 + 40.0) * 1024.0 + 2 * (10.0 * 2.0 + 4.0) * 1024.0
    assert got["cd_pass"]["bytes_per_pass"] == pytest.approx(per_pass)
    # a second workload is added beside the first
    monkeypatch.setattr(sys, "argv", ["pmc_traffic.py", "--workload", "toy2", "--fetch", str(tmp_path / "f"),
                                      "--write", str(tmp_path / "w")])
    pmc_traffic.main()
    assert set(json.load(open(out))) == {"toy", "toy2"}
