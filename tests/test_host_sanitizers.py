"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer: the library's scheduler (everything of the library
that runs on the CPU besides table building) and the CPU oracle are compiled with the host compiler, linked with a
sweep program (tests/sanitize/sweep.cpp) that drives random instances through both and cross-checks them, and run.
The sanitizers turn any out-of-bounds access, use after free, signed overflow or misaligned access into a failure."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.timeout(600)
def test_scheduler_and_oracle_under_asan_ubsan(tmp_path):
    if not (shutil.which("g++") and shutil.which("gcc")):
        pytest.skip("no host compiler")
    inc = ["-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2502_11058_amd", "csrc")]
    objs = []
    for cmd, src, obj in (
        (["gcc", "-std=c11", "-ffp-contract=off", "-fopenmp"], os.path.join(ROOT, "oracle", "plsgd_oracle.c"), "oracle.o"),
        (["g++", "-std=c++17"] + inc, os.path.join(ROOT, "paper_2502_11058_amd", "csrc", "ddp_schedule.cpp"), "schedule.o"),
        (["g++", "-std=c++17"] + inc, os.path.join(ROOT, "tests", "sanitize", "sweep.cpp"), "sweep.o"),
    ):
        o = str(tmp_path / obj)
        r = subprocess.run(cmd + SAN + ["-Wall", "-Wextra", "-c", src, "-o", o], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        objs.append(o)
    exe = str(tmp_path / "sweep")
    r = subprocess.run(["g++"] + SAN + ["-fopenmp"] + objs + ["-o", exe, "-lm"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe, "400"], capture_output=True, text=True, env=env, timeout=500)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitizer sweep ok" in r.stdout
