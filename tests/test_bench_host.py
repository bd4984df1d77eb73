"""Host-side pieces of the measurement (CPU only): bench.py's arguments and byte accounting, the profile summary
script and the traffic file that bench.py reads back."""
import csv
import importlib
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
bench = importlib.import_module("bench")


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout == ""


def test_bench_lines_and_their_bytes():
    assert bench.algo_config("topk") == ("topk", 10000, 0)
    assert bench.algo_config("topk-0.1") == ("topk", 1000, 0)
    assert bench.algo_config("topk-even") == ("topk", 10000, 0)
    assert bench.algo_config("dgc") == ("dgc", 1000, 0) and bench.algo_config("dgc-sampled") == ("dgc", 1000, 10000)
    D, W = 25557032, 8
    # every operand once: EF-Sign reads g and p, writes p and one bit; the sum reads W bits and writes a float
    assert bench.ALGO_BYTES["efsign_compress"](D, W, 0.0) == pytest.approx((4 + 4 + 4 + 1 / 8) * D)
    assert bench.ALGO_BYTES["dense_decompress"](D, W, 0.0) == pytest.approx((W / 8 + 4) * D)
    assert bench.ALGO_BYTES["sparse_accum"](D, W, 0.01) == pytest.approx(12.0 * D)
    assert bench.ALGO_BYTES["sparse_decompress"](D, W, 0.01) == pytest.approx((4 + 8 * 0.01 * W) * D)
    e = bench.call_entry("topk", D, W, 80e-6, 32e-6)
    assert e["algorithmic_GBps"] == pytest.approx(((12 + 0.08) + (4 + 0.64)) * D / 112e-6 * 1e-9)
    assert e["roofline_frac"] == pytest.approx(e["algorithmic_GBps"] / 8000.0)
    assert e["gradient_GBps"] == pytest.approx(4 * D / 112e-6 * 1e-9)


def write_csv(path, header, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(header)
        w.writerows(rows)


def test_profile_summary_scales_the_counters_and_writes_the_traffic_file(tmp_path, monkeypatch):
    """FETCH_SIZE counts 2 KiB units here (the copy of 262144 KiB reads 131072), WRITE_SIZE KiB: a kernel that
    fetches 1000 and writes 500 units moved 2000 KiB + 500 KiB."""
    k = "void mc::sign_compress_k<0, true>(mc::GroupView, float*)"
    pmc_header = ["Correlation_Id", "Dispatch_Id", "Grid_Size", "Kernel_Name", "Counter_Name", "Counter_Value"]
    write_csv(tmp_path / "f.csv", pmc_header, [[1, 1, 131072, "__amd_rocclr_copyBuffer", "FETCH_SIZE", 131072.0],
                                               [2, 2, 6240 * 256, k, "FETCH_SIZE", 1000.0], [3, 3, 6240 * 256, k, "FETCH_SIZE", 1000.0]])
    write_csv(tmp_path / "w.csv", pmc_header, [[1, 1, 131072, "__amd_rocclr_copyBuffer", "WRITE_SIZE", 262144.0],
                                               [2, 2, 6240 * 256, k, "WRITE_SIZE", 400.0], [3, 3, 6240 * 256, k, "WRITE_SIZE", 600.0]])
    write_csv(tmp_path / "s.csv", ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
              [[k, 2, 100000, 50000.0, 100.0, 49000, 51000, 1.0]])
    (tmp_path / "cmds.txt").write_text("rocprofv3 ... -- python3 bench.py\n")
    out, traffic = tmp_path / "summary.txt", tmp_path / "traffic.txt"
    r = subprocess.run([sys.executable, "-m", "paper_2103_15195_amd.profile_summary", "--stats", str(tmp_path / "s.csv"),
                        "--fetch", str(tmp_path / "f.csv"), "--write", str(tmp_path / "w.csv"), "--out", str(out), "--traffic", str(traffic),
                        "--title", "t", "--workload", "w", "--commands-file", str(tmp_path / "cmds.txt")], cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    text = out.read_text()
    assert "mc::sign_compress_k<0, true>" in text and "50.00" in text and "scale 2.0000" in text
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(traffic))
    t = bench.read_traffic()
    assert t == {"efsign_compress": pytest.approx((2000 + 500) * 1024)}      # the name the library's own profiler uses


def test_committed_traffic_file_covers_the_kernels_the_roofline_can_name():
    t = bench.read_traffic()
    for slot in bench.ALGO_BYTES:
        assert slot in t and t[slot] > 0
    # measured traffic of the streaming kernels stays within 10 % of the algorithmic bytes (else: wasted re-reads)
    D, W = 25557032, 8
    for slot in ("efsign_compress", "sparse_accum", "dense_decompress"):
        assert 0.98 < t[slot] / bench.ALGO_BYTES[slot](D, W, 0.01) < 1.10, slot
