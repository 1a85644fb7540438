"""paper_2511_10333_amd/profile_summary.py on small hand-made rocprofv3 CSVs: the calibration factor,
the per-launch means, the kernel-name folding and the line bench.py reads must come out as computed
by hand."""
import csv
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEAD = ["Correlation_Id", "Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]


def _write(folder, rows):
    os.makedirs(folder, exist_ok=True)
    with open(os.path.join(folder, "c_counter_collection.csv"), "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(HEAD)
        for i, (kernel, counter, value) in enumerate(rows):
            w.writerow([i, kernel[1], kernel[0], counter, value])


def test_traffic_summary_scales_by_the_copy_calibration(tmp_path):
    copy = ("copy_kernel(float*)", 1)
    # a 1 GiB copy that FETCH_SIZE reads as 524288 KiB (two bytes per counted byte) and WRITE_SIZE as 1048576
    _write(tmp_path / "cal_f", [(copy, "FETCH_SIZE", 524288.0)])
    _write(tmp_path / "cal_w", [(copy, "WRITE_SIZE", 1048576.0)])
    full = "void edgc::k_pass_p_deferred_full<1, 4, true, false, 8>(edgc::Group)"
    # two launches; the second one's counter arrives in two rows (two shader engines): summed per dispatch
    _write(tmp_path / "f", [((full, 1), "FETCH_SIZE", 1000.0), ((full, 2), "FETCH_SIZE", 500.0),
                            ((full, 2), "FETCH_SIZE", 1500.0), (("void edgc::k_chol(edgc::Group, unsigned int)", 3), "FETCH_SIZE", 10.0)])
    _write(tmp_path / "w", [((full, 1), "WRITE_SIZE", 300.0), ((full, 2), "WRITE_SIZE", 500.0)])
    out = tmp_path / "t.md"
    r = subprocess.run([sys.executable, "-m", "paper_2511_10333_amd.profile_summary", "traffic", "--workload", "w", "--rank", "8",
                        "--fetch", str(tmp_path / "f"), "--write", str(tmp_path / "w"), "--cal-fetch", str(tmp_path / "cal_f"),
                        "--cal-write", str(tmp_path / "cal_w"), "--out", str(out)], cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    text = out.read_text()
    # mean fetch = (1000 + 2000) / 2 = 1500 KiB x 2, mean write = 400 KiB x 1 -> 3400 KiB
    want = 3400 * 1024
    line = [l for l in text.splitlines() if l.startswith("traffic_bytes_per_launch k_pass_p_deferred ")]
    assert len(line) == 1 and abs(float(line[0].split()[-1]) - want) < 1.0     # the whole-tile kernel under the pass's name
    assert "traffic_bytes_per_launch k_chol 2.048000e+04" in text               # 10 KiB x 2, no writes counted

    sys.path.insert(0, ROOT)
    import bench
    (tmp_path / "traffic_probe_r8.md").write_text(text)
    got = bench.traffic_from_profile("probe", 8, "k_pass_p_deferred", folder=str(tmp_path))
    assert got[0] == want


def test_counters_summary_separates_launches_that_did_nothing(tmp_path):
    k = "void edgc::k_hist<float, 4, 1024>(edgc::EntGroup)"
    _write(tmp_path / "c", [((k, 1), "FETCH_SIZE", 1000.0), ((k, 2), "FETCH_SIZE", 2.0), ((k, 3), "FETCH_SIZE", 3000.0)])
    out = tmp_path / "c.md"
    r = subprocess.run([sys.executable, "-m", "paper_2511_10333_amd.profile_summary", "counters", "--dir", str(tmp_path / "c"),
                        "--title", "t", "--out", str(out)], cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    row = [l for l in out.read_text().splitlines() if l.startswith("| `k_hist<float, 4, 1024>`")]
    assert row == ["| `k_hist<float, 4, 1024>` | 2 | 1 | 2000 |"]      # two live launches, one idle, mean of the live ones
