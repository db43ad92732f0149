"""The CPU oracle against what the paper and the mathematics fix (no GPU, no HIP library)."""
import pytest

import oracle_pins


@pytest.mark.parametrize("pin", oracle_pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin()
