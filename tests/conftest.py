import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def repo_root():
    return ROOT


@pytest.fixture
def tuning():
    """Switches on the library's development switch for the test, so that the LINFUSION_* environment
    variables it sets (forced kernel routes, poll limit) are looked at; off again afterwards."""
    import paper_2409_02097_amd as lf
    lf.linfusion_set_tuning(True)
    yield
    lf.linfusion_set_tuning(False)


def pytest_terminal_summary(terminalreporter):
    """The largest result-relative gradient errors the run met (tests/parity.py: check_gradients)."""
    from tests import parity
    if parity.REL_L2_SEEN:
        terminalreporter.write_line("largest relative L2 error of a gradient tensor beyond its half ulp: " + ", ".join(
            f"{d} {n} {v:.2e}" for (d, n), v in sorted(parity.REL_L2_SEEN.items())))
