"""Command-line contract of the two benchmark scripts, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*argv):
    return subprocess.run([sys.executable, *argv], cwd=ROOT, capture_output=True, text=True, timeout=120)


@pytest.mark.parametrize("script", ["bench.py", "bench_table1.py"])
def test_help_renders(script):
    r = run(script, "--help")
    assert r.returncode == 0, r.stderr
    assert "usage" in r.stdout


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("bench.py", "--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
