"""The CPU oracle against what the paper's equations and plain mathematics fix (CPU only)."""
import numpy as np
import pytest

import oracle
from oracle_pins import BIGLA_PINS, BWD_PINS, GP_PINS, LOC_PINS


@pytest.mark.parametrize("pin", BIGLA_PINS, ids=lambda p: p.__name__)
def test_bigla_pin(pin):
    pin(oracle.bigla)


@pytest.mark.parametrize("pin", LOC_PINS, ids=lambda p: p.__name__)
def test_locality_pin(pin):
    pin(oracle.locality_gate)


@pytest.mark.parametrize("pin", GP_PINS, ids=lambda p: p.__name__)
def test_gate_producer_pin(pin):
    pin(oracle.gate_producer)


@pytest.mark.parametrize("pin", BWD_PINS, ids=lambda p: p.__name__)
def test_bigla_bwd_pin(pin):
    pin(oracle.bigla_bwd)


def test_gate_producer_feeds_bigla():
    """The produced log gates are valid inputs of the token mixer: <= 0, and with huge negative
    pre-activations in one direction that direction dies (only the own-token term survives)."""
    r = np.random.default_rng(5)
    B, L, D, H, dk, dv = 1, 6, 8, 2, 4, 3
    x = r.standard_normal((B, L, D))
    w1 = r.standard_normal((D, 16)) / 3
    w2 = r.standard_normal((16, 2 * H * dk))
    bias = np.concatenate([np.zeros(H * dk), np.full(H * dk, -1e5)])      # backward gates ~ 0
    gf, gb = oracle.gate_producer(x, w1, w2, H, dk, bias)
    assert np.all(gf <= 0) and np.all(gb < -1e3)
    q, k = r.standard_normal((2, B, H, L, dk))
    v = r.standard_normal((B, H, L, dv))
    out = oracle.bigla(q, k, v, gf, gb)
    only_fwd = oracle.bigla(q, k, v, gf, np.full_like(gb, -1e9))
    assert np.allclose(out, only_fwd, rtol=0, atol=1e-12)


def test_block_chain_limits():
    """The chained block output against what its definition fixes: with the gate closed
    (logits -> -inf) it is the token mixer's output, with the gate open the convolution's, and in
    between it moves along the segment between the two by exactly G (Section 4.2.2)."""
    r = np.random.default_rng(11)
    B, H, Hg, Wg, dk, dv = 2, 2, 3, 4, 3, 5
    L = Hg * Wg
    q, k = r.standard_normal((2, B, H, L, dk))
    gf, gb = -np.abs(r.standard_normal((2, B, H, L, dk))) / 4
    v, x, z = r.standard_normal((3, B, H, L, dv))
    w = r.standard_normal((H * dv, 3, 3))
    bias = r.standard_normal(H * dv)
    mixer = oracle.bigla(q, k, v, gf, gb)
    conv = oracle.locality_gate(x, w, np.full_like(z, 800.0), np.zeros_like(x), Hg, Wg, bias)
    closed = oracle.bigla_locality(q, k, v, gf, gb, x, w, np.full_like(z, -800.0), Hg, Wg, bias)
    opened = oracle.bigla_locality(q, k, v, gf, gb, x, w, np.full_like(z, 800.0), Hg, Wg, bias)
    assert np.array_equal(closed, mixer)
    assert np.array_equal(opened, conv)
    out = oracle.bigla_locality(q, k, v, gf, gb, x, w, z, Hg, Wg, bias)
    G = 1.0 / (1.0 + np.exp(-z))
    assert np.allclose(out - mixer, G * (conv - mixer), rtol=0, atol=1e-12)
    # the conv input is x, not the mixer's value tensor
    other = oracle.bigla_locality(q, k, v, gf, gb, x + 1.0, w, z, Hg, Wg, bias)
    assert not np.allclose(other, out)


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
