"""The plain-C program under examples/ (built by `python -m paper_2510_08525_amd.build` with the host compiler) drives
the library through include/rlkv.h alone - HIP runtime calls for memory, no Python objects behind the pointers -
and checks three decode steps of a mixed-head cache against softmax attention written out on the host."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plain_c_program_runs_the_path(gpu_device):
    binary = os.path.join(ROOT, "examples", "c_abi_decode")
    if not os.path.exists(binary):
        # (the build step makes it; a tree that arrives without it gets the one-second host compile here)
        from paper_2510_08525_amd import build

        build.build_example(verbose=False)
    res = subprocess.run([binary], capture_output=True, text=True, timeout=100)
    assert res.returncode == 0, res.stdout + res.stderr
    lines = res.stdout.strip().splitlines()
    assert lines[-1] == "OK" and sum(l.startswith("step ") for l in lines) == 3
    assert "lengths 43 43" in res.stdout
