"""Host-side checks of bench.py's command line (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env=e, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0
    assert "one-GPU" in r.stderr + r.stdout and "--gpus 1" in r.stderr + r.stdout
    assert not r.stdout.strip().startswith("{")  # no result line


def test_a_multi_rank_launch_is_refused_too():
    r = run_bench("--gpus", "1", env={"WORLD_SIZE": "2", "RANK": "0"})
    assert r.returncode != 0
    assert "one-GPU" in r.stderr + r.stdout
