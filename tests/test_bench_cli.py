"""Host-side checks of the benchmark's command line (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_nothing_committed_reads_the_scratch_folder_or_the_reference():
    """Product, tests and benchmark must not depend on working files or on the paper's text at run time."""
    bad = []
    for base, dirs, files in os.walk(ROOT):
        dirs[:] = [d for d in dirs if d not in (".git", "_work", "gpurun_out", "_build", "__pycache__", ".pytest_cache")]
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".c")) and f != os.path.basename(__file__):
                text = open(os.path.join(base, f), errors="replace").read()
                if "_work/" in text or "/root/reference" in text:
                    bad.append(os.path.join(base, f))
    assert not bad, bad
