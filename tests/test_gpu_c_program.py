"""The C ABI used the way a C program uses it: examples/step_from_c.c (plain C99, the HIP runtime's C
API, no Python in the process) places a state with ma_arena_create, runs ma_optimizer_step and
checks every element against the closed form of the first AdamW update."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "paper_2505_23254_amd", "step_from_c")


def test_c_program_steps_and_matches_the_closed_form():
    if not os.path.exists(EXE):
        pytest.skip("%s is not built (python -m paper_2505_23254_amd.build)" % EXE)
    run = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(run.stdout, run.stderr)
    assert run.returncode == 0, (run.returncode, run.stdout, run.stderr)
    lines = run.stdout.strip().splitlines()
    assert lines[-1] == "OK" and "0 of 3000007 elements off" in lines[-2] and "overflow 0" in lines[-2]
