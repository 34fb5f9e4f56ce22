"""The HIP kernel sources compiled for the host and run on a CPU emulation of the GPU's
execution model (tests/emu), in lockstep with the oracle: checks index arithmetic, control
flow and bounds (the arena sits between guard pages and starts out filled with garbage)
without a GPU.  The smallest legal model (d = 64, one head), where two of a workgroup's four
waves have no k-steps of a linear map at all; one case with 40 rows and two layers (32 x 32
units of QKV and FFN1 with a ragged second row block, per-layer advance of the descriptor table); one with 72 rows
(the kernel variant for 65 to 255 rows); one with 256 rows (the many-row kernel: 128 x 128 and 64 x 64 units with
their 16-byte pieces, whole-head attention units of two pairs); and the failure path of a step kernel that gave up
at a grid barrier (error word raised from the host); and models whose logits are all NaN (no arg-max, no draft
lists: the step must stay inside its buffers)."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "emu"))

pytestmark = pytest.mark.skipif(not os.path.exists("/opt/rocm/llvm/bin/clang++"), reason="needs ROCm's clang++")


@pytest.fixture(scope="module")
def emu_lib(tmp_path_factory):
    import emulate
    out = tmp_path_factory.mktemp("emu")
    lib = emulate.build(str(out))
    yield lib
    shutil.rmtree(str(out), ignore_errors=True)


@pytest.mark.parametrize("dtype", ["bf16", "fp32", "bf16-40rows", "bf16-72rows", "bf16-256rows", "bf16-giveup", "bf16-nan", "fp32-nan"])
def test_emulated_step_matches_oracle(emu_lib, dtype):
    r = subprocess.run([sys.executable, os.path.join(HERE, "emu", "run_case.py"), emu_lib, dtype],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=600, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
    assert ("recovered" if dtype == "bf16-giveup" else "stayed in bounds" if dtype.endswith("-nan") else "compared") in r.stdout
