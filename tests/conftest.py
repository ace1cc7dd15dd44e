import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    """How the 16-bit attention outputs of this run stood against the flat 2e-3 bar (see util.py)."""
    try:
        import util
    except Exception:
        return
    for name, st in sorted(util.STATS.items()):
        terminalreporter.write_line(
            "attention parity, %s outputs: %d heads compared with the oracle, %d above a flat 2e-3 relative L2 "
            "(each within the rounding of the exact result + 3e-4), worst head %.3e (%s)"
            % (name, st["heads"], st["above_2e-3"], st["worst"], st["worst_case"]))
