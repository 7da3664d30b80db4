"""The CPU oracle against its pins (no GPU).  See tests/pins.py for what each pin fixes."""
import pytest

import oracle
import pins


@pytest.fixture(scope="module")
def lib():
    return oracle.load()


@pytest.mark.parametrize("check", pins.ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(lib, check):
    check(lib)
