import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    """Parity reports of the whole-tensor tests (mismatch counts), shown for passing runs too."""
    from tests import harness
    if harness.REPORT_LINES:
        terminalreporter.write_sep("-", "parity reports")
        for line in harness.REPORT_LINES:
            terminalreporter.write_line(line)
