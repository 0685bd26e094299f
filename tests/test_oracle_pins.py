"""The CPU oracle against its pins (no GPU).  See pins.py for what each pin fixes."""
import os

import pytest

import pins


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(orc, pin):
    pin(orc)


def test_golden_exact_grid_fixture(orc):
    path = os.path.join(os.path.dirname(__file__), "golden", "sec2_4_exact_grid.txt")
    lines = [ln for ln in open(path).read().splitlines() if ln.strip() and not ln.startswith("#")]
    assert len(lines) == 4
    pins.pin_exact_grid_examples(orc, lines)
