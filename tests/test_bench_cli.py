"""bench.py's argument handling that needs no GPU."""
import os
import subprocess
import sys

from conftest import ROOT


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert run.returncode == 2
    assert "ONE GPU" in run.stderr and run.stdout.strip() == ""


def test_world_size_from_the_launcher_is_refused_too():
    env = dict(os.environ, WORLD_SIZE="4", RANK="0")
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                         timeout=120, env=env)
    assert run.returncode == 2 and "ONE GPU" in run.stderr
