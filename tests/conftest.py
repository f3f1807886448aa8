import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _oracle_progress_notes():
    """Where a run is watched through the files under gpurun_out/, the oracle's minutes-long calls leave notes there."""
    out = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(out):
        from oracle import oracle
        oracle.load("f64").set_progress_file(os.path.join(out, "oracle_progress.log"))
    yield


@pytest.fixture(scope="session")
def orc():
    from oracle import oracle
    return oracle.load("f64")


@pytest.fixture(scope="session")
def orc32():
    from oracle import oracle
    return oracle.load("f32")
