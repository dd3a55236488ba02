"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_profile_summary_names_its_command_and_kernel():
    text = open(os.path.join(ROOT, "profiles", "grad_stream_C3-lsq-n32-d4096.txt")).read()
    assert "rocprofv3 --kernel-trace --stats" in text and "bench.py" in text
    assert "grad_stream_kernel" in text and "traffic-bytes-per-launch:" in text
