"""Pins of the oracle's backward-side additions: the GELU derivatives, the data gradient taken
through an activation, and the bias gradient.  None of these is in the paper's Algorithm 1 (which
stops at the three products); they are the standard steps around them, pinned to mathematics:
finite differences of the activation itself, the identity g'(x) + g'(-x) = 1 that follows from
g(x) - g(-x) = x, textbook values of the normal density and CDF, limits, and brute force."""
import math
from fractions import Fraction

import numpy as np
import pytest

import axo_synth as syn
import oracle

XS = [-6.0, -3.0, -1.5, -0.75, -0.1, 0.0, 0.1, 0.5, 1.0, 2.0, 3.5, 6.0]


def py_gelu_erf(x):
    return 0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0)))


def py_gelu_tanh(x):
    return 0.5 * x * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


@pytest.mark.parametrize("d,f", [(oracle.dgelu_erf, py_gelu_erf), (oracle.dgelu_tanh, py_gelu_tanh)])
def test_derivative_matches_finite_differences_of_the_activation(d, f):
    for x in XS:
        h = 1e-5
        fd = (f(x - 2 * h) - 8 * f(x - h) + 8 * f(x + h) - f(x + 2 * h)) / (12 * h)  # 4th-order central difference
        assert abs(d(x) - fd) < 2e-10, (x, d(x), fd)


@pytest.mark.parametrize("d", [oracle.dgelu_erf, oracle.dgelu_tanh])
def test_derivative_identities_and_limits(d):
    assert d(0.0) == 0.5
    for x in XS:
        assert abs(d(x) + d(-x) - 1.0) < 1e-15      # from g(x) - g(-x) = x
    assert abs(d(12.0) - 1.0) < 1e-12 and abs(d(-12.0)) < 1e-12
    # the derivative dips below zero left of the minimum of the activation and exceeds one right of it
    assert d(-1.0) < 0.0 < d(-0.5) and d(1.0) > 1.0


def test_exact_form_against_textbook_normal_values():
    # Phi(1) = 0.8413447460685429, phi(1) = 0.24197072451914337 (standard normal table)
    assert abs(oracle.dgelu_erf(1.0) - (0.8413447460685429 + 0.24197072451914337)) < 1e-15
    # the two forms agree to the accuracy of the tanh approximation
    for x in XS:
        assert abs(oracle.dgelu_erf(x) - oracle.dgelu_tanh(x)) < 2e-3


def test_dgrad_through_activation_is_product_times_derivative():
    M, Kl, Nl = 9, 7, 11
    dY, W, P = (syn.normal_bf16(3, 0, (M, Nl), 1.0), syn.normal_bf16(3, 1, (Kl, Nl), 0.3),
                syn.normal_bf16(3, 2, (M, Kl), 1.5))
    plain = oracle.fc_dgrad(dY, W)
    for act, d in ((oracle.EPI_BIAS_GELU_TANH, oracle.dgelu_tanh), (oracle.EPI_BIAS_GELU_ERF, oracle.dgelu_erf)):
        got = oracle.fc_dgrad_act(dY, W, P, act)
        Pf = syn.bf16_bits_to_f64(P)
        want = plain * np.vectorize(d)(Pf)
        assert np.array_equal(got, want)
        rows = [8, 0, 3]
        assert np.array_equal(oracle.fc_dgrad_act(dY, W, P, act, rows=rows), want[rows])
    # a pre-activation far to the right passes the gradient through, far to the left blocks it
    big = syn.f32_to_bf16_bits(np.full((M, Kl), 20.0, dtype=np.float32))
    assert np.allclose(oracle.fc_dgrad_act(dY, W, big, oracle.EPI_BIAS_GELU_ERF), plain, rtol=1e-12)
    neg = syn.f32_to_bf16_bits(np.full((M, Kl), -20.0, dtype=np.float32))
    assert np.abs(oracle.fc_dgrad_act(dY, W, neg, oracle.EPI_BIAS_GELU_TANH)).max() < 1e-12


def test_bias_grad_brute_force_and_adjoint():
    M, Nl = 13, 10
    dY = syn.normal_bf16(4, 0, (M, Nl), 1.0)
    got = oracle.bias_grad(dY)
    vals = syn.bf16_bits_to_f64(dY)
    for n in range(Nl):
        exact = sum(Fraction(float(vals[t, n])) for t in range(M))
        assert got[n] == float(exact)
    # adjoint of the broadcast: <Y + 1 b^T, dY> - <Y, dY> = <b, colsum(dY)>
    b = syn.bf16_bits_to_f64(syn.normal_bf16(4, 1, (1, Nl), 1.0)[0])
    assert abs(np.sum(np.tile(b, (M, 1)) * vals) - np.dot(b, got)) < 1e-12
    # wgrad with a column of ones as X is the bias gradient
    ones = syn.f32_to_bf16_bits(np.ones((M, 1), dtype=np.float32))
    assert np.allclose(oracle.fc_wgrad(ones, dY)[0], got, rtol=0, atol=1e-13)
