"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_work_model_and_digest():
    sys.path.insert(0, ROOT)
    import bench
    from paper_1912_11040_amd import workloads as W
    assert abs(bench.conv_flop_per_sample(16000) - 152.0) < 1.0        # the transform's nominal flop count
    assert abs(bench.conv_flop_per_sample(32768) - 166.0) < 1.0
    w = W.tiny()
    work = bench.stage_work(w, n_images=1.0e6)
    assert work["rir"] == ("alu", 12.0e6)
    assert work["mel"][0] == "hbm" and work["mel"][1] == 4.0 * w.total * 2 + 4.0 * 40 * 8 * 98
    r = bench.roofline_for("rir", work, ms=1.0)
    assert r["peak"] == 78.6 and abs(r["frac"] - 12.0e6 / 1e-3 / 1e12 / 78.6) < 1e-12
    d = bench.kernel_source_digest()
    assert len(d) == 16 and d == bench.kernel_source_digest()
