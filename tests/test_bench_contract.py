"""CPU-only checks of bench.py's command line: it measures one GPU's share and says so when asked for more."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, env=e)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    r = _run(env={"WORLD_SIZE": "4"})
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_help_lists_the_shapes():
    r = _run("--help")
    assert r.returncode == 0
    for word in ("--shape", "team", "zigzag", "dit", "--config", "--steps", "--warmup"):
        assert word in r.stdout
