"""Pins for oracle/activation.py (the activation between fc1 and fc2 of the feed-forward block)."""
import numpy as np
from scipy.special import erf

from oracle import activation as A


def test_special_values_and_symmetry():
    assert A.gelu_tanh(0.0) == 0.0
    assert abs(A.gelu_tanh(10.0) - 10.0) < 1e-12 and abs(A.gelu_tanh(-10.0)) < 1e-12
    x = np.linspace(-8, 8, 4001)
    assert np.allclose(A.gelu_tanh(x) - A.gelu_tanh(-x), x, atol=1e-14)          # tanh is odd
    assert A.gelu_tanh_grad(0.0) == 0.5
    assert abs(A.gelu_tanh_grad(10.0) - 1.0) < 1e-9 and abs(A.gelu_tanh_grad(-10.0)) < 1e-9
    # the one hand value that fixes both constants: x = 1 -> 0.5 (1 + tanh(0.7978845608 * 1.044715))
    assert abs(A.gelu_tanh(1.0) - 0.5 * (1.0 + np.tanh(0.7978845608028654 * 1.044715))) < 1e-15
    assert abs(A.gelu_tanh(1.0) - 0.841191990608276) < 1e-12


def test_close_to_the_gaussian_cdf_form():
    """x Phi(x) is what the tanh form approximates; their distance is below 5e-4 everywhere (a wrong
    constant in either factor breaks this by orders of magnitude)."""
    x = np.linspace(-6, 6, 24001)
    exact = 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))
    d = np.abs(A.gelu_tanh(x) - exact)
    assert d.max() < 5e-4 and d.max() > 1e-4                                     # an approximation, not the exact form
    exact_grad = 0.5 * (1.0 + erf(x / np.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)
    assert np.abs(A.gelu_tanh_grad(x) - exact_grad).max() < 2e-3


def test_derivative_against_finite_differences():
    x = np.linspace(-7, 7, 2801)
    h = 1e-5
    num = (A.gelu_tanh(x + h) - A.gelu_tanh(x - h)) / (2 * h)
    assert np.abs(num - A.gelu_tanh_grad(x)).max() < 1e-9
