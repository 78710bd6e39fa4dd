"""The CPU oracle against its pins (no GPU)."""
import pytest

from oracle_pins import ALL_PINS


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda f: f.__name__)
def test_pin(orc, pin):
    pin(orc, orc.load())


def test_oracle_rejects_bad_shapes(orc):
    S = orc.Shape
    import numpy as np
    for bad in (S(0, 1, 1, 4, 4, 1, 1), S(1, 1, 1, 1, 1, 1, 1, 3, 1, 0), S(1, 1, 1, 4, 4, 1, 1, 3, 0, 1),
                S(1, 1, 1, 4, 4, 1, 1, 3, 1, -1), S(1, 1, 1, 4, 4, 0, 1)):
        with pytest.raises(ValueError):
            orc.conv_factored(bad, np.zeros(1), np.zeros(1), np.zeros(1), np.zeros(1))
