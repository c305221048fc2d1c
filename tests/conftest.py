import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: test needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_terminal_summary(terminalreporter):
    from tests import parity_util
    if parity_util.PARITY_LOG:
        terminalreporter.section("parity against the CPU oracle")
        for line in parity_util.PARITY_LOG:
            terminalreporter.write_line(line)
