"""TEST INFRASTRUCTURE ONLY -- gate predictor of SSA in plain fp64 numpy.

Paper, Sec. "Spatial Sparse Attention", text after eq. (4): the gating score of each module is obtained by a
linear layer followed by a sigmoid applied to the input features.  Reading: one linear layer d_model -> 3*H_q with
bias, output laid out [N, H_q, 3] in the branch order (cmp, slc, win) of the attention entry points.
Backward is the chain rule.  Nothing here is shared with the HIP library.
"""
from __future__ import annotations

import numpy as np


def gate_forward(x, w, b):
    """x [N, Dm], w [Dm, J], b [J] -> gates [N, J] = sigmoid(x w + b)."""
    z = np.asarray(x, np.float64) @ np.asarray(w, np.float64) + np.asarray(b, np.float64)
    return 1.0 / (1.0 + np.exp(-z))


def gate_backward(x, w, gates, dgates):
    """Gradients of sum(dgates * gates) given the forward result ``gates`` (the backward entry point takes the
    gates tensor, it does not recompute it): (dx [N, Dm], dw [Dm, J], db [J])."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w, np.float64)
    g = np.asarray(gates, np.float64)
    dz = np.asarray(dgates, np.float64) * g * (1.0 - g)
    return dz @ w.T, x.T @ dz, dz.sum(axis=0)
