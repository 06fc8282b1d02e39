"""CPU-side checks of the benchmark driver's contract: one GPU only, and the scripts fail loudly
without a GPU instead of falling back to anything."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, *args], cwd=ROOT, capture_output=True, text=True, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("bench.py", "--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_defaults_name_the_headline_workload():
    sys.path.insert(0, ROOT)
    import bench
    old = sys.argv
    sys.argv = ["bench.py"]
    try:
        args = bench.parse()
    finally:
        sys.argv = old
    assert args.gpus == 1 and args.workload == "headline_4k" and args.steps >= 1 and args.warmup >= 0
    from paper_2603_18567_amd.workloads import WORKLOADS
    wl = WORKLOADS[args.workload]
    assert (wl.T, wl.k, wl.hq, wl.hkv, wl.d, wl.dtype) == (4096, 7, 32, 8, 128, "bf16")


def test_no_gpu_means_an_error_not_a_fallback():
    import torch
    if torch.cuda.is_available():
        return   # on a GPU machine the benchmark itself is the test
    r = run("bench.py", "--steps", "1", "--warmup", "0", "--no-cpu-baseline")
    assert r.returncode != 0 and "metric" not in r.stdout
