"""The CPU oracle against what the paper's equations and plain mathematics fix (CPU only)."""
import numpy as np
import pytest

import oracle
from oracle_pins import BIGLA_PINS, LOC_PINS


@pytest.mark.parametrize("pin", BIGLA_PINS, ids=lambda p: p.__name__)
def test_bigla_pin(pin):
    pin(oracle.bigla)


@pytest.mark.parametrize("pin", LOC_PINS, ids=lambda p: p.__name__)
def test_locality_pin(pin):
    pin(oracle.locality_gate)


def test_thread_count_does_not_change_result():
    r = np.random.default_rng(0)
    q, k, gf, gb = (r.standard_normal((3, 2, 33, 8)) for _ in range(4))
    v = r.standard_normal((3, 2, 33, 5))
    gf, gb = -np.abs(gf), -np.abs(gb)
    a = oracle.bigla(q, k, v, gf, gb, nthreads=1)
    b = oracle.bigla(q, k, v, gf, gb, nthreads=4)
    assert np.array_equal(a, b)


def test_bad_shapes_rejected():
    q = np.zeros((1, 1, 4, 2))
    with pytest.raises(ValueError):
        oracle.bigla(q, np.zeros((1, 1, 4, 3)), np.zeros((1, 1, 4, 2)), q, q)
    with pytest.raises(ValueError):
        oracle.locality_gate(q, np.zeros((2, 3, 3)), q, q, 3, 2)
