"""The repo-level entry points run on the GPU the way the driver runs them."""
import pytest

pytestmark = pytest.mark.gpu


def test_smoke_entry_point_runs():
    import __graft_entry__
    __graft_entry__.smoke()
