"""The CPU oracle against what the mathematics, a library routine and the paper's walk-through fix."""
import os

import pytest

import oracle
from tests import oracle_pins as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def lib():
    from oracle import build
    return oracle.load(build.build(force=True))


@pytest.mark.parametrize("pin", P.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(lib, pin):
    pin(lib)


def test_slo_buffer_trace(lib):
    P.pin_slo_buffer_trace(lib, os.path.join(GOLDEN, "slo_buffer_trace.txt"))


def test_inflation_walkthrough(lib):
    P.pin_inflation_walkthrough(lib, os.path.join(GOLDEN, "inflation_walkthrough.txt"))
