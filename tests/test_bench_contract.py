"""Host-side contract of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    # one GPU is what this build runs on: any other count exits before anything touches a device
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode == 2
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_default_arguments_fit_the_contract():
    sys.path.insert(0, ROOT)
    import bench
    argv, sys.argv = sys.argv, ["bench.py"]
    try:
        args = bench.parse()
    finally:
        sys.argv = argv
    assert args.gpus == 1 and args.steps >= 1 and args.warmup >= 0
