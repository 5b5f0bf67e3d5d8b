"""The boundary from plain C: a C99 program that includes ``include/elsa.h``, links ``libelsa.so`` and
calls what needs no GPU (sizes, options, status strings, a dry-run plan and argument errors)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB_DIR = os.path.join(ROOT, "paper_2604_23798_amd")


def test_header_is_plain_c99_and_a_c_program_can_call_the_library(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    assert os.path.exists(os.path.join(LIB_DIR, "libelsa.so")), "build the library first (__graft_entry__.build())"
    exe = str(tmp_path / "c_caller")
    rocm_lib = "/opt/rocm/lib"
    subprocess.check_call([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c_caller.c"), "-o", exe, "-L", LIB_DIR, "-lelsa",
                           "-Wl,-rpath," + LIB_DIR, "-Wl,-rpath," + rocm_lib, "-Wl,-rpath-link," + rocm_lib])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "c caller: ok" in r.stdout, r.stdout + r.stderr
