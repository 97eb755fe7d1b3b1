"""The oracle against its pins (CPU only).  See oracle_pins.py for what each pin rests on."""
import pytest

import oracle_pins


@pytest.fixture(scope="module")
def api():
    return oracle_pins.OracleApi()


@pytest.mark.parametrize("pin", oracle_pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(api, pin):
    pin(api)
