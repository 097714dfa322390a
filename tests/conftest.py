import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    gu = sys.modules.get("tests.gpu_util") or sys.modules.get("gpu_util")
    worst = getattr(gu, "WORST", None) if gu else None
    if worst:
        terminalreporter.write_line("largest max-abs attention error compared, per GPU test:")
        for name, e in sorted(worst.items()):
            terminalreporter.write_line(f"  {e:.3e}  {name}")
