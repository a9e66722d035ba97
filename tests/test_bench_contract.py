"""bench.py on a machine without a GPU: the parts of its contract that need none."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, env=e,
                          timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout.strip() == ""
    r = run(env={"WORLD_SIZE": "4"})
    assert r.returncode == 2 and "single-GPU" in r.stderr


def test_help_lists_the_workloads():
    r = run("--help")
    assert r.returncode == 0
    for w in ("powerlaw", "stencil", "spmm", "bcsr_spmv", "bcsr_spmm", "mttkrp", "dcsr"):
        assert w in r.stdout
