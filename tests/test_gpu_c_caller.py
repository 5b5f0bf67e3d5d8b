"""GPU parity from plain C: tests/c_gpu_caller (built beforehand by tests/build_c_gpu_caller.py) allocates
with the HIP runtime, calls libelsa.so and checks against the C oracle; no Python object crosses the boundary."""
import os
import subprocess

import pytest

from tests import gpu_util as G

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_gpu_caller")


def test_c_program_runs_the_hot_path_and_matches_the_oracle():
    if not G.have_gpu():
        pytest.skip("no GPU")
    if not os.path.exists(EXE):              # normally built beforehand by __graft_entry__.build()
        from tests import build_c_gpu_caller
        build_c_gpu_caller.build()
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(r.stdout)
    assert r.returncode == 0 and "c gpu caller: ok" in r.stdout, r.stdout + r.stderr
