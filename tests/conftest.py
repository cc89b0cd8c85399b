"""Shared pytest setup: marker registration, build-if-missing, import path."""
import os
import sys

import pytest

# the library reads this switch once, at its first launch: with it the CNNMEM_* knobs that some tests use to
# force every kernel variant are live (they are dead in a process started without it)
os.environ["CNNMEM_KNOBS"] = "1"

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _built_libraries():
    """Load what is built; build when nothing is there or when a source is newer than the library."""
    import oracle
    oracle.build()
    from paper_1610_03618_amd import build as hip_build
    if hip_build.stale():
        hip_build.build()
    yield


def pytest_collection_modifyitems(config, items):
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
