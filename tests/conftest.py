import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests never run where no device is visible, whatever -m says.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Codes the HIP path placed one level off the oracle's float64 rule at a bucket boundary
    (each verified as such by the test that counted it), per test and in total."""
    pu = sys.modules.get("tests.parity_utils")
    if pu is None or not pu.BAND_COUNTS:
        return
    tr = terminalreporter
    tr.section("quantiser codes at a bucket boundary (one level off the float64 rule; 0 differ elsewhere)")
    band = elems = 0
    for test, (b, n) in pu.BAND_COUNTS.items():
        tr.write_line("%9d of %11d  (budget %5d)  %s" % (b, n, pu.code_band_budget(n), test))
        band += b
        elems += n
    tr.write_line("%9d of %11d  = %.2e of the codes checked (bar: 1e-5)" % (band, elems, band / max(elems, 1)))
