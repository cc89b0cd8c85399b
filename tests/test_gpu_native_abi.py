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
