"""Host-side checks of bench.py's command-line contract (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=120, env={**os.environ, **(env or {})})


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout.strip() == ""
    r = _run(env={"WORLD_SIZE": "4"})
    assert r.returncode == 2 and "single-GPU" in r.stderr


def test_the_flags_the_driver_passes_are_accepted():
    r = _run("--gpus", "1", "--steps", "3", "--warmup", "1", "--help")
    assert r.returncode == 0 and "--steps" in r.stdout and "--warmup" in r.stdout and "--gpus" in r.stdout
