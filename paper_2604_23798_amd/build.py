"""Build libelsa.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libelsa.so")
SOURCES = ["elsa_api.hip", "elsa_fwd_mfma.hip", "elsa_fwd_mfma_f16.hip", "elsa_fwd_fma.hip", "elsa_fwd_small.hip", "elsa_fwd_decode.hip", "elsa_combine.hip",
           "elsa_fwd_dv.hip", "elsa_fwd_dv_f16.hip", "elsa_probe.hip"]
HOST_SOURCES = ["elsa_plan.cpp"]       # plain C++ (launch planning): also built under sanitizers by a CPU test
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         # per-kernel registers, scratch (spill) bytes and occupancy, kept as _build/<source>.resources.txt
         "-Rpass-analysis=kernel-resource-usage"]
RESOURCES = os.path.join(HERE, "_build", "kernel_resources.txt")


def _hipcc():
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.sep not in c or os.path.exists(c):
            return c
    return "hipcc"


def _resource_table(remarks):
    """(mangled name, VGPRs, AGPRs, scratch bytes per lane, waves per SIMD) per kernel from hipcc's resource remarks."""
    import re
    rows, cur = [], None
    for line in remarks:
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = {"name": m.group(1)}
            rows.append(cur)
            continue
        for key, pat in (("vgpr", r" VGPRs: (\d+)"), ("agpr", r"AGPRs: (\d+)"), ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"),
                         ("occ", r"Occupancy \[waves/SIMD\]: (\d+)")):
            m = re.search(pat, line)
            if m and cur is not None:
                cur[key] = int(m.group(1))
    return [(r["name"], r.get("vgpr", -1), r.get("agpr", -1), r.get("scratch", -1), r.get("occ", -1)) for r in rows]


def build_library(verbose: bool = False) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o").replace(".cpp", ".o"))
        cmd = [hipcc, *(HOST_FLAGS if src in HOST_SOURCES else FLAGS), "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        remarks = [l for l in r.stderr.splitlines() if "kernel-resource-usage" in l]
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
        usage[src] = _resource_table(remarks)
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    usage = {}
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES + HOST_SOURCES))
    with open(RESOURCES, "w") as f:            # one line per kernel: source, mangled name, VGPRs, AGPRs, scratch bytes per lane, waves per SIMD
        for src in SOURCES:
            for row in usage[src]:
                f.write("%s %s\n" % (src, " ".join(str(x) for x in row)))
    tmp = LIB + ".tmp.%d" % os.getpid()
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
