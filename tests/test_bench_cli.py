"""Host-only checks of bench.py's command line: this build drives one GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    e = dict(os.environ)
    e.pop("WORLD_SIZE", None)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, env=e,
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr + r.stdout
    assert not any(line.startswith("{") for line in r.stdout.splitlines())   # no bench line


def test_a_multi_rank_launch_is_refused():
    r = _run(env={"WORLD_SIZE": "2", "RANK": "0"})
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr + r.stdout
