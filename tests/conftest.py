import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def toy_oracle():
    from tests import helpers
    return helpers.make_oracle(helpers.W.TOY_RING)


def pytest_runtest_logreport(report):
    """A GPU run is watched for output: every finished GPU test leaves one unbuffered line on stderr (pytest's own
    progress dots can sit in a pipe's buffer for the whole run)."""
    if report.when == "call" and "gpu" in report.keywords:
        sys.__stderr__.write(f"[gpu-test] {report.nodeid} {report.outcome} {report.duration:.1f}s\n")
        sys.__stderr__.flush()
