"""bench.py's command line: what it refuses, and that it never falls back to the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + list(args), capture_output=True, text=True,
                          timeout=300, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""                      # no result line


def test_without_a_gpu_there_is_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible here")
    r = run("--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "no GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_single_pair_goes_with_the_train_row_only():
    import torch
    if torch.cuda.is_available():
        pytest.skip("checked on the host side only")
    # the option is parsed before any device work; an unknown value is an argparse error
    r = run("--single-pair", "both")
    assert r.returncode != 0 and "invalid choice" in r.stderr
