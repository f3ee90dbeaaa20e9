"""bench.py's refusals, which need no GPU: more than one GPU is not what this build runs on, and --slabs needs --layers."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_slabs_need_layers():
    r = run("--slabs", "3")
    assert r.returncode == 2
    assert "--slabs needs --layers" in r.stderr and r.stdout.strip() == ""
    r = run("--config", "c4_paged", "--layers", "12", "--slabs", "4")   # 48 layers: more than the configuration has
    assert r.returncode == 2
