"""bench.py's command line contract that can be checked without a GPU: more than one GPU is refused with a message
(this build runs on one), option combinations that make no sense are refused, and without a GPU the run says so."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, cwd=ROOT, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_option_combinations():
    r = _bench("--smooth-k", "--format", "mx")
    assert r.returncode != 0 and "nvfp4" in r.stderr


def test_without_a_gpu_the_run_says_so():
    import torch
    if torch.cuda.is_available():
        return
    r = _bench("--steps", "1", "--warmup", "0", "--cpu-seconds", "0")
    assert r.returncode != 0 and "no GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line from a run that measured nothing
