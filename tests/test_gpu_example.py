"""The usage example that ships with the package runs and checks itself."""
import pytest

pytestmark = pytest.mark.gpu


def test_example_runs():
    from paper_2411_01611_amd import example
    assert example.main() < 1e-5
