"""The profile summary tool against small hand-made rocprofv3 CSV files: per-kernel statistics, counter
readings scaled by the reference copies of the same run, and the traffic lines bench.py reads back."""
import csv
import json
import os
import re

from paper_2601_09212_amd import profile_summary as ps


def _write(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)


def _raw(tmp_path, steps=20):
    raw = str(tmp_path / "raw")
    _write(os.path.join(raw, "trace", "host", "t_kernel_stats.csv"),
           ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
           [["void csd::row_stats_kernel<1, false, 2, 4, true, false>(csd::KArgs)", 100, 16000000, 160000, 80.0, 150000, 170000, 1.0],
            ["void csd::sequence_masses_kernel<1, false, true, 4, false>(csd::KArgs)", 50, 1250000, 25000, 6.0, 24000, 26000, 1.0],
            ["csd::read_probe_kernel(uint4 const*)", 10, 1800000, 180000, 9.0, 170000, 190000, 1.0],
            ["void at::native::vectorized_elementwise_kernel<4>(int)", 5, 1000, 200, 0.1, 100, 300, 1.0]])
    head = ["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]
    for sub, counter, unit in (("fetch", "FETCH_SIZE", 2048.0), ("write", "WRITE_SIZE", 1024.0)):
        rows, d = [], 0
        for _ in range(5):                                    # the reference copies: 2^30 bytes each way
            d += 1
            rows.append([d, "void at::native::vectorized_elementwise_kernel<4>(int)", counter, (1 << 30) / unit])
        for _ in range(steps):
            d += 1
            rows.append([d, "void csd::row_stats_kernel<1, false, 2, 4, true, false>(csd::KArgs)", counter,
                         (1000.0e6 if sub == "fetch" else 2.0e6) / unit])
            d += 1
            rows.append([d, "void csd::sequence_masses_kernel<1, false, true, 4, false>(csd::KArgs)", counter,
                         (100.0e6 if sub == "fetch" else 0.0) / unit])
        _write(os.path.join(raw, sub, "host", sub[0] + "_counter_collection.csv"), head, rows)
    with open(os.path.join(raw, "trace.log"), "w") as f:
        f.write("noise\n" + json.dumps({"value": 1.0, "ms_per_step": 0.2, "config": {"workload": "x"},
                                         "roofline": {"bound": "hbm", "frac": 0.5}}) + "\n")
    return raw


def test_summary_lines_and_scaling(tmp_path):
    raw = _raw(tmp_path)
    text = ps.summary("cfg5", raw, [], sq=False)
    # dominant kernel by total time (the read yardstick is not a candidate), bytes = fetch + write
    m = re.search(r"^traffic_bytes_per_launch:\s*(\S+)\s+([0-9.eE+]+)\s*$", text, flags=re.M)
    assert m and m.group(1) == "csd::row_stats_kernel" and abs(float(m.group(2)) - 1002.0e6) < 1.0
    m = re.search(r"^traffic_bytes_per_call:\s*([0-9.eE+]+)\s*$", text, flags=re.M)
    assert m and abs(float(m.group(1)) - 1102.0e6) < 1.0        # both kernels, once per call
    assert "bytes per unit from the reference copy: 2048.0" in text and "bytes per unit from the reference copy: 1024.0" in text
    assert "rocprofv3 --output-format csv --kernel-trace --stats" in text and "--pmc FETCH_SIZE" in text
    # runs that also call other entry points give no per-call figure
    assert "traffic_bytes_per_call" not in ps.summary("cfg5", raw, ["--lantern"], sq=False)
    assert "traffic_bytes" not in ps.summary("cfg5", raw, ["--draft-sampler"], sq=False, trace_only=True)


def test_bench_reads_the_summary_back(tmp_path, monkeypatch):
    import bench
    raw = _raw(tmp_path)
    prof = tmp_path / "profiles"
    prof.mkdir()
    (prof / "verify_cfg5_rocprofv3.md").write_text(ps.summary("cfg5", raw, [], sq=False))
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert abs(bench.measured_traffic("cfg5") - 1002.0e6) < 1.0
    assert abs(bench.measured_traffic("cfg5", per_call=True) - 1102.0e6) < 1.0
    assert bench.measured_traffic("cfg4") is None               # no summary: no figure
