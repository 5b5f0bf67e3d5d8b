"""Build tests/c_gpu_caller (plain C99, gcc): the hot path called with no Python in the process.
Run on the CPU beforehand (``__graft_entry__.build()`` does); the binary travels with the tree."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
EXE = os.path.join(HERE, "c_gpu_caller")


def build(rocm: str = "/opt/rocm") -> str:
    lib_dir = os.path.join(ROOT, "paper_2604_23798_amd")
    oracle_so = os.path.join(ROOT, "oracle", "_elsa_oracle.so")
    assert os.path.exists(os.path.join(lib_dir, "libelsa.so")) and os.path.exists(oracle_so), "build the library and the oracle first"
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-Wno-unused-parameter", "-Wno-unused-function",
           "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(rocm, "include"),
           os.path.join(HERE, "c_gpu_caller.c"), "-o", EXE,
           "-L", lib_dir, "-lelsa", "-L", os.path.dirname(oracle_so), "-l:_elsa_oracle.so", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           # found next to the tree wherever it is copied to
           "-Wl,-rpath,$ORIGIN/../paper_2604_23798_amd", "-Wl,-rpath,$ORIGIN/../oracle", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.check_call(cmd)
    return EXE


if __name__ == "__main__":
    print(build())
