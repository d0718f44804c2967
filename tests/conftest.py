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


def pytest_terminal_summary(terminalreporter):
    """Largest errors the GPU parity tests measured against each oracle (figures quoted in the design notes)."""
    try:
        from hs_common import STATS
    except Exception:
        return
    if STATS:
        terminalreporter.write_line("parity maxima: " + ", ".join(f"{k}={v:.3g}" for k, v in sorted(STATS.items())))
