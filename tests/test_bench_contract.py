"""bench.py's command-line contract, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_measured_traffic_is_tied_to_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    same = bench.sources_hash() == bench.MEASURED_SOURCES
    for stage in ("scan", "decode", "reconstruct", "resize"):
        t = bench.measured_traffic(2, stage)
        assert (t is not None) == same
        if same:
            assert t > 0
    # no counters were taken for these workloads
    assert bench.measured_traffic(3, "decode") is None
    assert bench.measured_traffic(5, "resize") is None


def test_algorithmic_bytes_of_one_known_image():
    sys.path.insert(0, ROOT)
    import bench

    class Info:
        width, height, sampling = 256, 256, 1
        mcu_cols, mcu_rows, blocks_per_mcu = 16, 16, 6
        entropy_bytes = 10000

    pr = dict(resize_short=256, crop_h=224, crop_w=224, out_dtype="f16")
    work, entropy = bench.algorithmic_bytes([Info()], pr)
    assert entropy == 10000
    assert work["scan"] == 10000
    # the crop reads source pixels 16 .. 239 of each axis: MCUs 1 .. 14 of 16
    assert work["reconstruct"] == 14 * 14 * (6 * 128 + 256 * 3)
    assert work["resize"] == 224 * 224 * 3 + 3 * 224 * 224 * 2
