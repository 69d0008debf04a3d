import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    """Reports how many first-token argmax comparisons were strict and how many fell inside the measured error."""
    mod = sys.modules.get("tests.gpu_util")
    if mod is None:
        return
    t = mod.ARGMAX_TALLY
    if t["identical"] + t["within_error"]:
        terminalreporter.write_line(f"first-token argmax vs oracle: {t['identical']} identical (strict), "
                                    f"{t['within_error']} with the oracle's top-2 gap inside twice the logit error "
                                    f"(GPU choice among the oracle's two best)")
