"""The CPU oracle against its pins (closed forms, library routines, brute force,
invariants, the paper's worked example).  CPU only."""
import pytest

from oracle import finch_oracle as O
from tests import oracle_pins


@pytest.mark.parametrize("pin", oracle_pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(O)
