"""The C ABI used from a plain C99 program (no Python, no torch): tests/native/abi_step.c runs one whole
decode step per dtype through hgca_hybrid_decode_step and checks it against the C oracle it links.  The
program is built by __graft_entry__.build() (tests/native/build_abi_step.py)."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "abi_step")


def test_plain_c_program_runs_the_step_and_agrees_with_the_oracle():
    assert os.path.exists(EXE), "tests/native/abi_step is not built: run __graft_entry__.build()"
    run = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(run.stdout, run.stderr, flush=True)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "abi_step: ok" in run.stdout
