"""The staging-slot pool of the search entry points, exercised on the host alone: the pool's
header knows nothing of HIP, so a small C++ program drives it with fake events from many threads
and checks that no slot is ever held by two calls at once and that no slot is handed out while
the work recorded behind its last use is pending."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_14881_amd", "csrc")
SRC = os.path.join(ROOT, "tests", "stage_pool_host_test.cpp")


@pytest.mark.parametrize("sanitize", [False, True])
def test_slots_have_one_owner_and_wait_for_their_last_use(tmp_path, sanitize):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "stage_pool_host_test")
    cmd = [cxx, "-std=c++17", "-O1", "-pthread", "-I", CSRC, SRC, "-o", exe]
    if sanitize:
        cmd[1:1] = ["-fsanitize=thread"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if sanitize and built.returncode != 0:
        pytest.skip("ThreadSanitizer runtime not available: " + built.stderr[-200:])
    assert built.returncode == 0, built.stderr
    # more threads than slots, so that calls also meet a pool with every slot owned
    run = subprocess.run([exe, "24" if not sanitize else "12", "3000"], capture_output=True, text=True, timeout=240)
    assert run.returncode == 0, run.stdout + run.stderr
    words = run.stdout.split()
    assert words[0] == "ok" and int(words[1]) == (24 if not sanitize else 12) * 3000
