"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, gcc / g++).

The library's planner (`csrc/planner.cpp`) and the oracle's C loops (`oracle/gdws_oracle.c`) are
compiled with `-fsanitize=address,undefined -fno-sanitize-recover=all` together with a small driver
each (`tests/host/`) that walks every routine over small irregular shapes; any report makes the
driver exit non-zero.  The sanitizer runtimes are linked statically so that the run does not depend
on the order of preloaded libraries.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
       "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           LD_PRELOAD="")


def build_and_run(tmp_path, compiler, sources, includes, expect):
    exe = str(tmp_path / "walk")
    cmd = [compiler] + SAN + [f"-I{i}" for i in includes] + sources + ["-o", exe, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=ENV)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert expect in r.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="no g++")
def test_planner_under_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2110_14871_amd", "csrc")
    build_and_run(tmp_path, "g++", ["-std=c++17", os.path.join(csrc, "planner.cpp"),
                                    os.path.join(ROOT, "tests", "host", "sanitize_planner.cpp")],
                  [csrc, os.path.join(ROOT, "include")], "planner sanitizer walk ok")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_oracle_c_under_sanitizers(tmp_path):
    build_and_run(tmp_path, "gcc", [os.path.join(ROOT, "oracle", "gdws_oracle.c"),
                                    os.path.join(ROOT, "tests", "host", "sanitize_oracle.c")],
                  [], "oracle sanitizer walk ok")
