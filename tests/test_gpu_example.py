"""The usage example that ships with the package runs and checks itself."""
import pytest

pytestmark = pytest.mark.gpu


def test_example_runs():
    from paper_2411_01611_amd import example
    assert example.main() < 1e-5


def test_example_lookahead_loop_runs():
    from paper_2411_01611_amd import example
    assert example.lookahead_loop() < 1e-6
