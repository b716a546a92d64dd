"""bench.py's command-line contract that can be checked without a GPU."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_nothing_committed_depends_on_the_working_folder():
    # sources, tests and the benchmark must not read or import anything under _work/
    bad = []
    for base, dirs, files in os.walk(ROOT):
        dirs[:] = [d for d in dirs if d not in (".git", "_work", "gpurun_out", "__pycache__", "_build")]
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h", ".c")) and f != os.path.basename(__file__):
                text = open(os.path.join(base, f), errors="replace").read()
                if re.search(r"_work(?![A-Za-z_])", text):
                    bad.append(os.path.join(base, f))
    assert not bad, bad
