"""The benchmark's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1",
                        "--warmup", "0"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_kernel_fingerprint_covers_existing_files():
    sys.path.insert(0, ROOT)
    import bench
    for name in bench.KERNEL_SOURCES:
        assert os.path.exists(os.path.join(ROOT, "paper_2506_11728_amd", "csrc", name)), name
    assert len(bench.kernel_fingerprint()) == 16
