"""The CPU oracle against everything the paper and arithmetic fix (no GPU)."""
import pytest

from pins import ALL_PINS


@pytest.mark.parametrize("name,pin", ALL_PINS, ids=[n for n, _ in ALL_PINS])
def test_pin(oracle, name, pin):
    pin(oracle)
