import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def rs():
    """The HIP library binding; GPU tests fail loudly if it is not built."""
    from paper_2605_28640_amd import binding
    binding.load()
    return binding


class _Knobs:
    """RATSPARSE_* tuning variables for one test: the library reads its environment once per
    process, so every change is followed by the re-read hook."""

    def __init__(self, monkeypatch, lib):
        self._mp, self._lib = monkeypatch, lib

    def setenv(self, name, value):
        self._mp.setenv(name, value)
        self._lib.ratsparse_debug_reload_knobs()

    def delenv(self, name):
        self._mp.delenv(name, raising=False)
        self._lib.ratsparse_debug_reload_knobs()


@pytest.fixture
def knobs(rs, monkeypatch):
    k = _Knobs(monkeypatch, rs.load())
    yield k
    monkeypatch.undo()
    rs.load().ratsparse_debug_reload_knobs()
