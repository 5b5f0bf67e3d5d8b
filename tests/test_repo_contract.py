"""Host-side checks of the repository's own rules: the product path never touches the oracle, the
benchmark refuses more than one GPU, and the documented file map matches the tree."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _read(path):
    with open(os.path.join(ROOT, path), encoding="utf-8") as f:
        return f.read()


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_23798_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".hpp", ".h")):
                text = _read(os.path.relpath(os.path.join(dirpath, name), ROOT))
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), name
                assert "elsa_oracle" not in text, name
    assert "oracle" not in _read("include/elsa.h")
    # and the oracle does not reach into the product
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith((".py", ".c")):
            text = _read(os.path.join("oracle", name))
            assert "paper_2604_23798_amd" not in text and "libelsa" not in text, name


def test_only_tests_smoke_and_the_cpu_baseline_use_the_oracle():
    bench = _read("bench.py")
    uses = [m.start() for m in re.finditer(r"^\s*import oracle", bench, re.M)]
    assert uses, "the cpu_baseline leg times the oracle"
    for pos in uses:                       # every import sits inside a baseline function or its branch of main
        head = bench[:pos]
        fn = re.findall(r"^def (\w+)\(", head, re.M)[-1]
        assert fn in ("spot_parity", "cpu_baseline_varlen", "main")      # spot_parity is the timed oracle leg (cpu_baseline calls it)
    entry = _read("__graft_entry__.py")
    assert entry.count("import oracle") == 2           # build() compiles it, smoke() checks against it


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and not r.stdout.strip()


def test_documented_files_exist():
    design = _read("DESIGN.md")
    for path in re.findall(r"`((?:paper_2604_23798_amd|tests|oracle|include|profiles)/[\w./]+)`", design):
        if "*" in path or path.endswith("/"):
            continue
        assert os.path.exists(os.path.join(ROOT, path)), path
    srcs = _read("paper_2604_23798_amd/build.py")
    for name in re.findall(r'"(elsa_\w+\.hip)"', srcs):
        assert os.path.exists(os.path.join(ROOT, "paper_2604_23798_amd", "csrc", name)), name
        assert name in design or name.replace(".hip", "") in design, "the design document does not mention " + name


def test_every_gpu_test_module_is_marked():
    tests = os.path.join(ROOT, "tests")
    for name in sorted(os.listdir(tests)):
        if name.startswith("test_gpu") and name.endswith(".py"):
            assert "pytestmark = pytest.mark.gpu" in _read(os.path.join("tests", name)), name
