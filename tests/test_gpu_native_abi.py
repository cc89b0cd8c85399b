"""The C ABI used from a plain C++ program: its own hipMalloc'd buffers and stream, no Python or PyTorch in the
process.  The program (tests/native/abi_parity.cpp) is compiled by ``__graft_entry__.build()`` and compares the
library with the oracle itself; this test only runs it and reports what it printed."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
BINARY = os.path.join(HERE, "native", "abi_parity.bin")


def test_native_program_matches_the_oracle():
    assert os.path.exists(BINARY), f"{BINARY} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`"
    run = subprocess.run([BINARY], capture_output=True, text=True, timeout=300)
    print(run.stdout)
    print(run.stderr)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-2000:]
    assert "all checks passed" in run.stdout


def test_native_launch_cost_program_runs():
    """Host cost per call and eager steps against graph replays (measurement; the bound here is only a guard
    against a launch path that regresses to many times the cost of a replay)."""
    binary = os.path.join(HERE, "native", "launch_cost.bin")
    assert os.path.exists(binary), f"{binary} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`"
    run = subprocess.run([binary], capture_output=True, text=True, timeout=300)
    print(run.stdout)
    print(run.stderr)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-2000:]
    last = run.stdout.strip().splitlines()[-1]
    assert last.startswith("eager / graph:")
    ratios = [float(t) for t in last.replace("eager / graph:", "").replace("and", " ").split()]
    assert all(r < 3.0 for r in ratios), last
