"""The smoke entry point itself, so that a change which breaks it fails the GPU suite."""
import pytest

pytestmark = pytest.mark.gpu


def test_smoke_entry_point_runs():
    import __graft_entry__

    __graft_entry__.smoke()
