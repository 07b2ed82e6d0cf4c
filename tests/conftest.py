import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_terminal_summary(terminalreporter):
    """Weight-gradient errors measured by the GPU parity tests (whole-tensor error scale)."""
    try:
        from gpu_util import DW_ERRORS
    except ImportError:
        return
    if DW_ERRORS:
        terminalreporter.write_line("weight-gradient errors against the oracle (max|err| / rms of the whole tensor):")
        for name, err in sorted(DW_ERRORS.items()):
            terminalreporter.write_line(f"  {name}: {err:.3e}")
