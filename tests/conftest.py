import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def ref():
    """The CPU oracle (built on first use)."""
    import oracle
    oracle.lib()
    return oracle


def pytest_terminal_summary(terminalreporter):
    """How close the GPU-vs-oracle fragment selections of this session came to a tie."""
    util = sys.modules.get("parity_util")
    if util is not None and util.SESSION_LOG.compared:
        terminalreporter.write_line(f"[selection parity] {util.SESSION_LOG}")
