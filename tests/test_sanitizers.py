"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only; the GPU code objects are not
instrumented): the oracle's C source with a condensed battery of its pins, and the library's launch
planner (plain C++, the same file the library links) over the documented shapes and a seeded random grid."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def _run(exe):
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)                 # the sanitizer runtime must come first in the library list
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    return subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)


def test_oracle_c_source_is_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.check_call([gcc, "-std=c99", "-Wall", "-Wextra", *SAN, "-static-libasan", "-ffp-contract=off",
                           os.path.join(ROOT, "oracle", "elsa_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitize.c"),
                           "-o", exe, "-lm"])
    r = _run(exe)
    assert r.returncode == 0 and "oracle under sanitizers: ok" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]


def test_launch_planner_is_clean_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "plan_sanitize")
    csrc = os.path.join(ROOT, "paper_2604_23798_amd", "csrc")
    subprocess.check_call([gxx, "-std=c++17", "-Wall", "-Wextra", *SAN, "-static-libasan", "-I", csrc,
                           os.path.join(csrc, "elsa_plan.cpp"), os.path.join(ROOT, "tests", "plan_sanitize.cpp"), "-o", exe])
    r = _run(exe)
    assert r.returncode == 0 and "planner under sanitizers: ok" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
