"""The C ABI driven from C++ alone: `paper_2604_26837_amd/examples/one_step.cpp` allocates with hipMalloc,
runs set-up and one decode step through `include/spin.h` and checks the output against dense attention over
the pages the library reports.  The test runs the program built beside libspin.so (as a child process)."""
import os
import subprocess

import pytest

from paper_2604_26837_amd import build

pytestmark = pytest.mark.gpu


def test_cpp_caller_runs_one_step_and_checks_it():
    if not os.path.exists(build.EXAMPLE_BIN):
        build.build_example()
    r = subprocess.run([build.EXAMPLE_BIN], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "one_step: ok" in r.stdout
