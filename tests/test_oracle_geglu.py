"""Pins of the oracle's gated activation out = a * GELU(b) (oracle.geglu).

The definition is the models' (the transformer feed-forward of the networks the paper
quantizes, Section 4.1), GELU(t) = t * Phi(t) with Phi the standard normal distribution
function.  Pinned against textbook values of Phi, an identity, the limits, a library
routine with a different implementation of Phi, and a case that tells the two halves of
the channel dimension apart.
"""
import numpy as np

import oracle


def _gelu_via_oracle(t):
    t = np.asarray(t, dtype=np.float32).reshape(-1, 1)
    y = np.concatenate([np.ones_like(t), t], axis=1)  # a = 1, b = t
    return oracle.geglu(y)[:, 0].astype(np.float64)


def test_textbook_values_of_the_normal_distribution_function():
    # Phi(0) = 1/2, Phi(1) = 0.8413447460685429, Phi(2) = 0.9772498680518208 (any table)
    got = _gelu_via_oracle([0.0, 1.0, -1.0, 2.0, -2.0])
    want = np.array([0.0, 0.8413447460685429, -(1.0 - 0.8413447460685429),
                     2.0 * 0.9772498680518208, -2.0 * (1.0 - 0.9772498680518208)])
    assert np.allclose(got, want.astype(np.float32), rtol=0, atol=1e-7)


def test_antisymmetric_part_is_half_the_argument():
    # Phi(t) + Phi(-t) = 1  =>  GELU(t) - GELU(-t) = t
    t = np.linspace(-6, 6, 241).astype(np.float32)
    g = _gelu_via_oracle(t)
    gm = _gelu_via_oracle(-t)
    assert np.allclose(g - gm, t.astype(np.float64), rtol=0, atol=5e-7)


def test_limits():
    big = _gelu_via_oracle([12.0, 40.0, -12.0, -40.0])
    assert big[0] == 12.0 and big[1] == 40.0
    assert abs(big[2]) < 1e-30 and big[3] == 0.0


def test_against_a_library_distribution_function():
    from scipy.special import ndtr  # a different implementation of Phi
    rng = np.random.default_rng(7)
    y = (3.0 * rng.standard_normal((64, 96))).astype(np.float32)
    got = oracle.geglu(y).astype(np.float64)
    a, b = y[:, :48].astype(np.float64), y[:, 48:].astype(np.float64)
    want = a * b * ndtr(b)
    assert np.allclose(got, want, rtol=2e-7, atol=1e-7)


def test_first_half_is_the_value_second_half_the_gate():
    # a = 2, b = 1 -> 2 * GELU(1) = 1.68269; the halves swapped would give GELU(2) = 1.95450
    y = np.array([[2.0, 1.0]], dtype=np.float32)
    out = oracle.geglu(y)
    assert out.shape == (1, 1)
    assert abs(float(out[0, 0]) - 2.0 * 0.8413447460685429) < 1e-6
    # channel c pairs with channel O/2 + c, not with its neighbour
    y = np.array([[1.0, 10.0, 0.0, 5.0]], dtype=np.float32)  # a = (1, 10), b = (0, 5)
    out = oracle.geglu(y)[0]
    assert out[0] == 0.0 and abs(float(out[1]) - 10.0 * 5.0 * 0.9999997133484281) < 1e-4
