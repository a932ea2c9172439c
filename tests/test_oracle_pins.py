"""The CPU oracle against what the paper's definition and mathematics fix
(section 3.2.1: softmax attention restricted to the sink + recent set)."""
import pytest

import oracle_pins as P


@pytest.mark.parametrize("pin", P.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin, oracle_lib):
    pin(None)
