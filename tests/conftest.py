import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(scope="session")
def built_library():
    """Requested by the tests that call the HIP library (the GPU parity tests and the ABI checks); the oracle's pins
    need neither the HIP toolchain nor the product package and do not request it.  The tests load the library that
    is built in-tree; only when there is none do they build it (hipcc cross-compiles without a GPU).  After a change
    to a source, build again before running the tests."""
    from paper_2105_14088_amd.build import LIB_PATH, build
    if not os.path.exists(LIB_PATH):
        build(force=True)
    return LIB_PATH


def pytest_terminal_summary(terminalreporter):
    """Coverage lines of the full-size GPU parity cases (restarts and orders compared with the oracle)."""
    util = sys.modules.get("gpu_util")
    lines = getattr(util, "SUMMARY", []) if util else []
    if lines:
        terminalreporter.section("full-size parity coverage")
        for line in lines:
            terminalreporter.write_line(line)
