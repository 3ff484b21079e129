"""bench.py's command line: the parts that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True,
                          text=True, timeout=300, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    for n in ("2", "8"):
        r = run("--gpus", n, "--steps", "1", "--warmup", "0")
        assert r.returncode != 0
        assert "ONE GPU" in r.stderr and "--gpus must be 1" in r.stderr
        assert r.stdout.strip() == ""                 # no JSON line for a run that did not happen


def test_unknown_workload_or_kind_is_an_argument_error():
    assert run("--kind", "nonsense").returncode == 2
    assert run("--bf16", "--f16", "--gpus", "3").returncode != 0
