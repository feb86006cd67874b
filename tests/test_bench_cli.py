"""bench.py's command line on a machine without a GPU: what must hold before any GPU work starts."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    """This build keeps all replicas in one GPU's memory: `--gpus N` with N > 1 must exit with a message that says so,
    before anything touches a device."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus must be 1" in r.stderr
    assert r.stdout.strip() == ""           # no JSON line of a run that did not happen


def test_unknown_workload_is_rejected_by_the_parser():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "cfg9"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "invalid choice" in r.stderr
