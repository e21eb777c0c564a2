import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_lib():
    from oracle import conv
    conv.build()
    return conv


@pytest.fixture
def knob(monkeypatch):
    """Set one of the library's TWN_* tuning overrides for the rest of the test: the library reads them once, so
    it is told to read them again after the change and after the change is undone."""
    from paper_1605_04711_amd import api

    def set_knob(name, value):
        monkeypatch.setenv(name, str(value))
        api.reload_env()

    yield set_knob
    monkeypatch.undo()
    api.reload_env()
