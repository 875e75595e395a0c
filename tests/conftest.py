import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests must never silently pass on a box without a GPU.
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """Achieved parity errors of this run against their bars (filled by util.close)."""
    try:
        from util import MARGINS
    except Exception:
        return
    if not MARGINS:
        return
    tr = terminalreporter
    tr.write_line("")
    tr.write_line("parity margins: worst achieved error (normwise | element-wise |got-ref|/(|ref|+16 rms)) against the bar")
    for key in sorted(MARGINS):
        tol, e_norm, e_elem, n = MARGINS[key]
        tr.write_line("  %-58s %9.2e | %9.2e  bar %7.1e  (%d tensors)" % (key[:58], e_norm, e_elem, tol, n))
