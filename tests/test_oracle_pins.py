"""The CPU oracle against its pins (no GPU): worked examples, exact rational
arithmetic, library special cases and invariants.  See tests/oracle_pins.py."""
import pytest

import oracle_pins


@pytest.mark.parametrize("check", oracle_pins.ALL_CHECKS, ids=lambda f: f.__name__)
def test_oracle_pin(check):
    check(None)
