"""CPU-only: the oracle against brute force, library routines, closed forms and worked values."""
import pytest

import pins


@pytest.mark.parametrize("check", pins.ALL_CHECKS, ids=lambda f: f.__name__)
def test_oracle_pin(oracle, check):
    check(oracle)
