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
    import oracle as _o
    _o.build()
    return _o


def pytest_terminal_summary(terminalreporter):
    """Diagnostics the GPU parity tests record (reported, not gated): distance to the exact oracle, to the
    rounding-faithful diagnostic oracle, worst 64-column block, elementwise check."""
    import util
    if util.DIAG_LINES:
        terminalreporter.write_sep("-", "parity diagnostics (max relative error, normwise; tolerance 2e-2 bf16 / 1e-5 fp32)")
        for line in util.DIAG_LINES:
            terminalreporter.write_line(line)
