import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI HIP library)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


def pytest_terminal_summary(terminalreporter):
    """What the GPU parity cases compared (rows, decisions, near-ties), also under -q."""
    import xsm_harness
    if xsm_harness.SUMMARY:
        terminalreporter.write_sep("-", "parity tallies (flagged = near-ties, not compared)")
        for line in xsm_harness.SUMMARY:
            terminalreporter.write_line(line)
