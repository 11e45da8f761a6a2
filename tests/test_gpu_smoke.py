"""The smoke entry point itself, so that it cannot rot unnoticed."""
import pytest

pytestmark = pytest.mark.gpu


def test_smoke_entry_point_runs_and_checks_against_the_oracle():
    import __graft_entry__ as g

    g.smoke()
