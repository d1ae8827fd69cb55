"""The CPU oracle against its pins (closed forms, library routines, brute force, finite differences,
the paper's invariants).  CPU only."""
import pytest

import oracle.ais_oracle as O
from tests import oracle_pins


@pytest.mark.parametrize("pin", oracle_pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(O)
