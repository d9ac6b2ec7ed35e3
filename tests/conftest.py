import os
import sys

import pytest

ROOT = os.path.abspath(os.path.join(os.path.dirname(__file__), ".."))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture
def tuning(monkeypatch):
    """Sets SPEC_VERIFY_* tuning switches for one test: the library reads its environment once,
    so the switches are re-read after every change and once more when the test is over."""
    from paper_2406_14066_amd import spec_verify as sv

    def set_switch(name, value):
        monkeypatch.setenv(name, str(value))
        sv.reload_env()

    yield set_switch
    monkeypatch.undo()
    sv.reload_env()
