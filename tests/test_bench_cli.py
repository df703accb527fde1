"""Host logic of bench.py that needs no GPU: one GPU only, and no result without one."""
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the behaviour of a machine without a GPU")
def test_no_gpu_means_an_error_and_no_result_line():
    """There is no CPU fall-back behind the bench: without a device it fails and prints no JSON."""
    r = _bench("--steps", "1", "--warmup", "1", "--no-cpu-baseline")
    assert r.returncode != 0
    assert "{" not in r.stdout


def test_shape_override_needs_one_workload_and_a_whole_number_of_blocks():
    r = _bench("--shape", "1,32,32,4096")
    assert r.returncode == 2 and "--only" in r.stderr and r.stdout.strip() == ""
    r = _bench("--only", "--workload", "llama7b_4bit", "--shape", "1,32,32,4100")
    assert r.returncode == 2 and "block size" in r.stderr
    r = _bench("--only", "--workload", "llama13b_mixed", "--shape", "1,40,40,4096")
    assert r.returncode == 2 and "append" in r.stderr
