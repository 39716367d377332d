import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import oracle as orc
    orc.lib()
    return orc


@pytest.fixture(autouse=True)
def _parity_report(request):
    """Names the running test for the error table that helpers.max_rel_err fills."""
    import helpers
    helpers.begin_report(request.node.name)
    yield
    helpers.begin_report(None)


def pytest_terminal_summary(terminalreporter):
    """Per test: the worst per-tensor error (the quantity the tolerances bound) and the worst
    element-wise relative error over the elements above 1e-3 of their tensor's maximum."""
    import helpers
    if not helpers.REPORT:
        return
    tr = terminalreporter
    tr.write_sep("-", "parity report: worst per-tensor error | worst element-wise relative error (|ref| > 1e-3 max) | tensors")
    for name, (err, elem, n) in helpers.REPORT.items():
        tr.write_line(f"{err:9.2e} | {elem:9.2e} | {n:3d} | {name}")
