"""CPU oracle for the Softmax op and its backprop -- TEST INFRASTRUCTURE ONLY.

The paper names softmax next to convolution as a kernel a backend supplies
(Sec. 4, the paragraph on the cuDNN transformer) and derives backward graphs by
autodiff of the forward ops (Sec. 3); it gives no formula, so the oracle is the
textbook definition, written out in fp64 with numpy:

    softmax(x)[i, j]      = exp(x[i, j]) / sum_k exp(x[i, k])              (last axis)
    softmax_bwd(y, dy)[i] = J(y[i])^T dy[i],  J = diag(y) - y y^T
                          = y[i] * (dy[i] - sum_k dy[i, k] y[i, k])

exp(x - m) / sum exp(x - m) equals the definition for every real m; taking
m = max_k x[i, k] keeps fp64 exp in range for any finite input, so the oracle
evaluates that form.  Inputs are finite.

Pins (tests/test_oracle_pins.py): closed forms (constant rows, two-element
rows = logistic function, arithmetic-progression rows = geometric series), the
unshifted definition on small inputs, scipy.special.softmax, shift invariance,
rows summing to one, the explicit Jacobian on small rows and central
differences for the backprop.
"""
from __future__ import annotations

import numpy as np


def softmax(x) -> np.ndarray:
    """Softmax over the last axis, fp64."""
    x = np.asarray(x, dtype=np.float64)
    m = x.max(axis=-1, keepdims=True)
    e = np.exp(x - m)
    return e / e.sum(axis=-1, keepdims=True)


def softmax_bwd(y, dy) -> np.ndarray:
    """Backprop of softmax over the last axis: y is the forward result, dy the delta of it."""
    y = np.asarray(y, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    assert y.shape == dy.shape
    s = (dy * y).sum(axis=-1, keepdims=True)
    return y * (dy - s)
