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


def test_missing_library_fails_loudly_and_there_is_no_fallback(tmp_path):
    env = dict(os.environ, DDLSIM_LIBRARY=str(tmp_path / "nowhere" / "libddlsim.so"))
    code = "import paper_1708_02188_amd as D\nD.ddl_ring_plan([2], 2, 8)\n"
    run = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True,
                         timeout=240, env=env)
    assert run.returncode != 0
    assert "ImportError" in run.stderr and "no fallback" in run.stderr
    # nothing in the package imports the oracle
    pkg = os.path.join(ROOT, "paper_1708_02188_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
