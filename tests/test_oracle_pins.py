"""The CPU oracle against its pins (no GPU). See tests/oracle_pins.py for what fixes each value."""
import pytest

import oracle_pins


@pytest.mark.parametrize("pin", oracle_pins.ALL_PINS, ids=lambda f: f.__name__)
def test_oracle_pin(pin):
    pin(None)
