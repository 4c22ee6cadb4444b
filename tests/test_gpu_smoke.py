"""The entry point's smoke run is part of the GPU suite, so that it cannot go stale unnoticed."""
import pytest

pytestmark = pytest.mark.gpu


def test_smoke_entry_point():
    import __graft_entry__ as entry
    entry.smoke()
