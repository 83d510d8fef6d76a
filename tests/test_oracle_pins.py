"""CPU-only: the float64 oracle against closed forms, autodiff of an unrolled
forward, finite differences, Theorem 1's Elman reduction and invariants."""
import pytest

import oracle
from oracle_pins import ALL_CHECKS


@pytest.mark.parametrize("check", ALL_CHECKS, ids=lambda c: c.__name__)
def test_oracle_pin(check):
    check(oracle.fwd, oracle.bwd)
