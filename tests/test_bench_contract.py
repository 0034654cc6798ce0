"""Host-side checks of bench.py's contract that need no GPU: more than one GPU is refused with a message, and
without a GPU the script says so instead of falling back to anything."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    env = dict(os.environ, HIP_VISIBLE_DEVICES="", CUDA_VISIBLE_DEVICES="")      # no GPU for this process
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, env=env,
                          timeout=300)


def test_more_than_one_gpu_is_refused():
    res = _run("--gpus", "2")
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_no_gpu_is_an_error_not_a_fallback():
    res = _run("--steps", "1", "--warmup", "0")
    assert res.returncode != 0
    assert "no GPU" in res.stderr and res.stdout.strip() == ""
