"""Host-side sanitizer tier: the planner and the CPU oracle compiled with AddressSanitizer and
UndefinedBehaviorSanitizer (gcc, CPU only) and driven by tests/sanitize/driver.cpp - a planner
fuzz over seeded shapes, metrics and limits, and the oracle's heap selection against its
written-out definition on tie-rich tiny inputs.  Any report aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="gcc not available")
def test_planner_and_oracle_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    oracle_o = tmp_path / "oracle.o"
    subprocess.run(["gcc", "-std=c11", "-fopenmp", "-ffp-contract=off", *san, "-c",
                    os.path.join(ROOT, "oracle", "knn_oracle.c"), "-o", str(oracle_o)], check=True)
    exe = tmp_path / "sanitize_driver"
    subprocess.run(["g++", "-std=c++17", "-fopenmp", *san,
                    os.path.join(ROOT, "tests", "sanitize", "driver.cpp"),
                    os.path.join(ROOT, "paper_2206_14148_amd", "csrc", "planner.cpp"),
                    str(oracle_o), "-lm", "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1",
               OMP_NUM_THREADS="2")
    env.pop("LD_PRELOAD", None)  # the sanitizer runtime has to come first in the link order
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitizer driver ok" in r.stdout
