"""The host-side planner, scheduler and work-item planning (plain C++, no GPU) built with AddressSanitizer and
UndefinedBehaviorSanitizer and driven by seeded random batches (tests/native/host_fuzz.cpp): memory safety plus the
structural guarantees of their outputs (every token in exactly one slice, valid segment tables, every chunk in exactly
one pipeline, checkpointing plans that fit their capacity in the timeline)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_21275_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_and_scheduler_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",  # linked in, so that nothing depends on the order of preloaded libraries
           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "native", "host_fuzz.cpp"),
           os.path.join(CSRC, "chunk_plan.cpp"), os.path.join(CSRC, "chunk_sched.cpp"), os.path.join(CSRC, "plan.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "sanitize" in r.stderr:
        pytest.skip("this g++ has no sanitizer runtime")
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe, "300"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert r.stdout.startswith("ok 300 cases")
