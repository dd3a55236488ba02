"""The context's pool of host threads (bookkeeping of many rounds) under ThreadSanitizer:
every job runs each of its shares exactly once, jobs of changing width follow one another on
the same threads, and an idle pool shuts down.  Host code only; needs g++."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("sanitizer", ["thread", "address,undefined"])
def test_host_pool_under_sanitizers(tmp_path, sanitizer):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "host_pool_check")
    build = subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-fsanitize=" + sanitizer,
                            "-I", os.path.join(ROOT, "paper_2212_08580_amd", "csrc"),
                            os.path.join(ROOT, "tests", "host_pool_check.cpp"), "-o", exe, "-lpthread"],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), run.stdout
