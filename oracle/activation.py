"""Activation between the two linear layers of the feed-forward block (Sec. 6 sparsifies both linears of
every FFN block; the appendix times that block).

Test infrastructure only (see the package header).

The paper does not name the activation.  Reading taken: the models whose layer shapes its experiments use
(GPT-2) apply GELU in its tanh form,

    gelu(x) = 0.5 x (1 + tanh( sqrt(2 / pi) (x + 0.044715 x^3) )),

so that is the activation between fc1 and fc2 here; its derivative is the analytic one.  float64.

Pinned (tests/test_oracle_activation.py): special values, the identity gelu(x) - gelu(-x) = x, closeness
to the exact Gaussian-CDF form x Phi(x) (scipy's erf) within the published error of the tanh form,
and the derivative against central finite differences and against the derivative of x Phi(x).
"""
import numpy as np

_K0 = np.sqrt(2.0 / np.pi)
_K1 = 0.044715


def gelu_tanh(x):
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + np.tanh(_K0 * (x + _K1 * x ** 3)))


def gelu_tanh_grad(x):
    """d gelu_tanh / dx."""
    x = np.asarray(x, dtype=np.float64)
    t = np.tanh(_K0 * (x + _K1 * x ** 3))
    du = _K0 * (1.0 + 3.0 * _K1 * x ** 2)
    return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * du
