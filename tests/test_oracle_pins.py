"""Run every pin of `oracle_pins.py` against the real CPU oracle.  CPU only."""
import pytest

import oracle_pins


@pytest.mark.parametrize("pin", oracle_pins.PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin()
