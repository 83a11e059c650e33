"""Host-side behaviour of bench.py that needs no GPU: more than one GPU is refused with a message (this build has
no collectives), and without a GPU the product path fails loudly instead of falling back to anything."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
    assert "{" not in r.stdout          # no result line


def test_help_lists_the_workload_switches():
    r = _run("--help")
    assert r.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--config", "--backward", "--mx", "--swiglu", "--quantize", "--launch-plan"):
        assert flag in r.stdout
