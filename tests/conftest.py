import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    """Largest error each kind of compared quantity reached in this run (relative to its scale)."""
    try:
        import parity
    except ImportError:
        return
    if parity.OBSERVED:
        terminalreporter.write_line("largest observed errors (relative to the tensor's scale):")
        for key, rel in sorted(parity.OBSERVED.items()):
            terminalreporter.write_line("  %-60s %.2e" % (key, rel))
