"""The library's host state machine (descriptor validation, closed-form ring tables) built for the
CPU with AddressSanitizer and UBSan and soaked with 10 000 seeded random append / reset calls per
ring shape against a naive ring simulation written in the harness; 4000 random descriptors go
through validation.  Any sanitizer report or table mismatch fails the run."""
import os
import shutil
import subprocess

import pytest


def test_ring_tables_soak_under_address_and_undefined_behaviour_sanitizers(repo_root, tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    src = os.path.join(repo_root, "tests", "host_soak", "ring_soak.cpp")
    exe = str(tmp_path / "ring_soak")
    build = subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror", "-fsanitize=address,undefined",
                            "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", src, "-o", exe],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)   # the sanitizer runtime must come first in the process
    run = subprocess.run([exe, "10000"], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "ring soak ok: 120000 random append/reset calls" in run.stdout
