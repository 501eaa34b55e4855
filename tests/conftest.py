import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle.build()
    return oracle


class _SwitchPatch:
    """pytest's monkeypatch, plus: the library reads its NGC_* environment switches once per process, so every
    change of one of them (and the undo at the end of the test) is followed by ngc_reload_switches()."""

    def __init__(self, mp):
        self._mp = mp
        self.touched = False

    def _reload(self, name):
        if str(name).startswith("NGC_"):
            import paper_1801_08058_amd as ng
            ng.ngc_reload_switches()
            self.touched = True

    def setenv(self, name, value, *a, **k):
        self._mp.setenv(name, value, *a, **k)
        self._reload(name)

    def delenv(self, name, *a, **k):
        self._mp.delenv(name, *a, **k)
        self._reload(name)

    def __getattr__(self, attr):
        return getattr(self._mp, attr)


@pytest.fixture
def monkeypatch(monkeypatch):
    p = _SwitchPatch(monkeypatch)
    yield p
    monkeypatch.undo()
    if p.touched:
        import paper_1801_08058_amd as ng
        ng.ngc_reload_switches()
