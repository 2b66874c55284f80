"""The CPU oracle against what the paper and mathematics fix (no GPU)."""
import pytest

import oracle
from oracle_pins import ALL_CHECKS, check_hand_example


@pytest.fixture(scope="module")
def lib():
    return oracle.load()


@pytest.mark.parametrize("check", ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(lib, check):
    check(lib)


def test_hand_example_f64(lib):
    check_hand_example(lib, dtype="f64")


def test_create_rejects_bad_arguments(lib):
    import numpy as np
    for (W, P, d, tau) in ((0, 4, 1, 1), (2, 4, -1, 1), (2, 4, 1, 0)):
        with pytest.raises((ValueError, AssertionError)):
            oracle.Oracle(W, P, d, tau, 0.1, 0.9, 0.0, np.zeros(max(P, 1)))
