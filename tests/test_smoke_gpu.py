"""The driver's smoke entry point, run as a GPU test so that a stale assertion in it is caught here."""
import pytest

pytestmark = pytest.mark.gpu


def test_graft_entry_smoke():
    import __graft_entry__ as g
    g.smoke()
