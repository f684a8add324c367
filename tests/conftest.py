import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_present():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


# Normalised max errors the parity tests measured, printed once at the end of the run (also under -q).
_PARITY = []


@pytest.fixture
def parity_record():
    def record(tag, err, tol):
        _PARITY.append((tag, float(err), float(tol)))
    return record


def pytest_terminal_summary(terminalreporter):
    if not _PARITY:
        return
    terminalreporter.write_line("normalised max error vs the CPU oracle (whole tensors):")
    for tag, err, tol in _PARITY:
        terminalreporter.write_line("  %-44s %.3e  (bar %.1e)" % (tag, err, tol))
