"""CPU test: the fp64 linear-layer checker against what the mathematics fixes (sections 2.1, 3.1)."""
import pytest

import oracle
from tests import linear_pin_checks


@pytest.mark.parametrize("check", linear_pin_checks.ALL_CHECKS, ids=lambda f: f.__name__)
def test_linear_pin(check):
    check(oracle.linear)


def test_index_outside_the_matrices_is_an_error():
    import numpy as np
    x = np.zeros((2, 4), np.uint16); w = np.zeros((3, 4), np.uint16)
    with pytest.raises(ValueError):
        oracle.linear(x, w, rows=[2])
    with pytest.raises(ValueError):
        oracle.linear(x, w, cols=[-1])
    with pytest.raises(ValueError):
        oracle.linear(x, np.zeros((3, 5), np.uint16))
