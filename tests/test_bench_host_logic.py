"""Host-side logic of the benchmark and of the profile summarizer (no GPU): the algorithmic byte counts
against the per-element formulas, the tracked traffic and clock readings, the one-GPU rule, and the
summarizer on small synthetic rocprofv3 output."""
import csv
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench                                                # noqa: E402
from paper_1804_08066_amd import rocprof_summary as rs      # noqa: E402


def test_algorithmic_bytes_follow_the_per_element_formulas():
    # quantize: 4 + b/8 + 4/bucket per element; update: W (b/8 + 4/bucket) + 8 per parameter
    n = 100_000_000
    for bits in (1, 2, 4, 8):
        for bucket in (128, 1024, 8192):
            nb = -(-n // bucket)
            assert bench.quantize_bytes(n, bits, bucket) == pytest.approx(n * (4 + bits / 8) + 4 * nb)
            for W in (8, 16):
                assert bench.aggregate_bytes(n, bits, bucket, W) == pytest.approx(W * (n * bits / 8 + 4 * nb) + 8 * n)
    # the headline point as the design notes quote it
    assert round(bench.quantize_bytes(n, 4, 1024) / 1e6, 2) == 450.39
    assert round(bench.aggregate_bytes(n, 4, 1024, 8) / 1e6, 1) == 1203.1


def test_traffic_comes_from_the_tracked_profile_and_only_for_its_workload():
    d = bench.measured_traffic(100_000_000, 8, 4, 1024)
    assert d is not None and d["commit"]
    algorithmic = bench.quantize_bytes(100_000_000, 4, 1024)
    assert 0.99 * algorithmic < d["quantize_wave_kernel"] < 1.05 * algorithmic
    assert bench.measured_traffic(100_000_000, 8, 2, 1024) is None
    assert bench.measured_traffic(1_000_000, 8, 4, 1024) is None


def test_load_clock_is_read_from_the_tracked_machine_state():
    mhz = bench.load_clock_mhz()
    assert mhz is not None and 500 < mhz <= 2400
    row = bench.alu_row("k", 0.1, 1e9)
    assert row["bound"] == "alu" and row["peak"] == pytest.approx(256 * 64 * 2.4e9 / 1e12)
    assert row["peak_at_load_clock"] == pytest.approx(256 * 64 * mhz * 1e6 / 1e12)
    assert row["frac_at_load_clock"] >= row["frac"]


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr


def test_kernel_names_are_told_apart():
    ns = "void mqg::(anonymous namespace)::"
    assert rs.short(ns + "requantize_wave_kernel<4, 1, 4, 4, false, true, 0, 4>(mqg::RequantArgs)") == "requantize_wave_kernel"
    assert rs.short(ns + "quantize_wave_kernel<8, 1, 4, 5, false>(mqg::QuantizeArgs)") == "quantize_wave_kernel"
    assert rs.short(ns + "requantize_minmax_tensor_kernel<256, false, true>(mqg::RequantArgs)") == "requantize_minmax_tensor_kernel"
    assert rs.short(ns + "quantize_tensors_cells_kernel<4, 8, false>(mqg::BatchQuantizeArgs)") == "quantize_tensors_cells_kernel"
    assert rs.short(ns + "range_finish_batch_kernel(mqg::TensorRangeBatch, unsigned int)") == "range_finish_batch_kernel"
    assert rs.short("__amd_rocclr_copyBuffer") == "plain copy (torch copy_)"
    assert rs.short("at::native::elementwise_kernel<...>") is None


def test_stats_summary_merges_template_instances(tmp_path):
    path = tmp_path / "stats_kernel_stats.csv"
    ns = "void mqg::(anonymous namespace)::"
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"])
        w.writerow([ns + "quantize_wave_kernel<8, 1, 4, 5, false>(mqg::QuantizeArgs)", 30, 0, 70000.0, 0, 68000, 90000, 0])
        w.writerow([ns + "quantize_wave_kernel<8, 1, 4, 8, false>(mqg::QuantizeArgs)", 10, 0, 74000.0, 0, 66000, 80000, 0])
        w.writerow(["at::native::something", 5, 0, 1.0, 0, 1, 1, 0])
    ks = rs.kernel_stats(str(path))
    assert list(ks) == ["quantize_wave_kernel"]
    calls, avg, lo, hi = ks["quantize_wave_kernel"]
    assert calls == 40 and avg == pytest.approx(71000.0) and (lo, hi) == (66000, 90000)
    out = tmp_path / "s.md"
    r = subprocess.run([sys.executable, "-m", "paper_1804_08066_amd.rocprof_summary", "stats", "--title", "t", "--cmd", "c",
                        "--csv", str(path), "--measured-at", "abc1234", "--out", str(out)], cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    text = out.read_text()
    assert "Measured at commit abc1234." in text and "| quantize_wave_kernel | 40 | 71000 | 66000 | 90000 |" in text


def test_traffic_summary_ends_with_the_line_the_benchmark_reads(tmp_path):
    def counters(name, copy_kib, q_kib, a_kib, path):
        with open(path, "w", newline="") as f:
            w = csv.writer(f)
            w.writerow(["Kernel_Name", "Counter_Name", "Counter_Value"])
            for k, v in (("__amd_rocclr_copyBuffer", copy_kib), ("mqg::quantize_wave_kernel<8>", q_kib),
                         ("mqg::aggregate_update_rows_kernel<2>", a_kib)):
                w.writerow([k, name, v])
                w.writerow([k, name, v])
    n = 1 << 20
    true_kib = 4.0 * n / 1024
    fetch, write = tmp_path / "f.csv", tmp_path / "w.csv"
    counters("FETCH_SIZE", true_kib / 2, 1000.0, 3000.0, fetch)     # the counter reads half the bytes
    counters("WRITE_SIZE", true_kib, 100.0, 4000.0, write)
    out = tmp_path / "t.md"
    r = subprocess.run([sys.executable, "-m", "paper_1804_08066_amd.rocprof_summary", "traffic", "--title", "t", "--cmd", "c1",
                        "--cmd", "c2", "--fetch", str(fetch), "--write", str(write), "--n", str(n), "--measured-at", "abc1234",
                        "--out", str(out)], cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    last = [ln for ln in out.read_text().splitlines() if ln.startswith("traffic_json:")]
    assert len(last) == 1
    d = json.loads(last[0][len("traffic_json:"):])
    assert d["commit"] == "abc1234" and d["workload"]["n"] == n
    assert d["quantize_wave_kernel"] == pytest.approx((2 * 1000.0 + 100.0) * 1024, rel=1e-6)
    assert d["aggregate_update_rows_kernel"] == pytest.approx((2 * 3000.0 + 4000.0) * 1024, rel=1e-6)
