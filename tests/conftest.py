import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def fc():
    """The HIP path's Python binding; fails loudly when the library is not built."""
    import paper_2501_04012_amd as pkg
    return pkg


def pytest_terminal_summary(terminalreporter):
    """Measured parity errors (HIP path against the oracle) of the tests that ran."""
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import util
    if not util.PARITY:
        return
    terminalreporter.write_sep("-", "measured parity errors")
    for test, values in util.PARITY:
        terminalreporter.write_line(test + ": " + ", ".join("%s=%.3e" % kv for kv in values.items()))
