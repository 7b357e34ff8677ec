"""TEST INFRASTRUCTURE ONLY -- the linear projections around SSA in plain fp64 numpy.

Paper: the attention of eq. (2)-(4) acts on query, key and value tokens obtained from the input features by linear
layers, as in any attention layer, and its result goes through an output projection (Implementation Details: DiT
blocks with hidden dimension 1024); the paper prints no formula for them.  Reading: y = x W^T + b with W stored
[d_out][d_in] (one row per output feature), bias optional.  Backward is the chain rule.  Nothing here is shared with
the HIP library.
"""
from __future__ import annotations

import numpy as np


def linear_forward(x, w, b=None):
    """x [N, d_in], w [d_out, d_in], b [d_out] or None -> y [N, d_out]."""
    y = np.asarray(x, np.float64) @ np.asarray(w, np.float64).T
    return y if b is None else y + np.asarray(b, np.float64)


def linear_backward(x, w, dy):
    """Gradients of sum(dy * y): (dx [N, d_in], dw [d_out, d_in], db [d_out])."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w, np.float64)
    dy = np.asarray(dy, np.float64)
    return dy @ w, dy.T @ x, dy.sum(axis=0)
