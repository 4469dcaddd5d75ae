import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests must never silently pass on a box without a GPU or without the built library.
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    # the margins the GPU parity checks were passed with (worst case over the run, per kind of check)
    try:
        import parity
    except Exception:
        return
    if not parity.OBSERVED:
        return
    terminalreporter.write_sep("-", "worst observed errors of the GPU parity checks")
    for kind, (value, what, bar) in sorted(parity.OBSERVED.items()):
        terminalreporter.write_line(f"{kind}: {value:.3e}  ({value / bar:.2%} of the bar; in: {what})")
