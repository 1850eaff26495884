"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one-GPU" in r.stderr or "one-GPU" in r.stdout
    assert "{" not in r.stdout          # no JSON line is printed for a run that did not happen


def test_bench_and_smoke_do_not_reach_outside_the_repository():
    """The GPU machine has no reference tree: nothing the driver runs there may name it."""
    for name in ("bench.py", "__graft_entry__.py"):
        src = open(os.path.join(ROOT, name)).read()
        assert "/root/reference" not in src and "_work/" not in src
