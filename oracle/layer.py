"""TEST INFRASTRUCTURE ONLY -- one full SSA attention layer in fp64: projections, gate predictor, attention, output
projection, chained from the oracles of the parts.

Paper: eq. (4) combines the three attention branches with gates "obtained by applying a linear layer followed by a
sigmoid activation to the input features"; queries, keys and values are linear projections of the same input features
and the result passes an output projection, as in any attention layer (Implementation Details: hidden dimension 1024,
grouped-query attention).  Reading: q = x Wq^T, k = x Wk^T, v = x Wv^T (optional biases), gates = sigmoid(x Wg + bg),
o = SSA(q, k, v, gates), y = o Wo^T (+ bo).  Backward is the chain rule with the selected sets held constant.
Nothing here is shared with the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from .gate import gate_backward, gate_forward
from .linear import linear_backward, linear_forward
from .ssa_oracle import ForwardResult, Oracle


@dataclass
class LayerWeights:
    wq: np.ndarray  # [Hq*d, Dm]
    wk: np.ndarray  # [Hkv*d, Dm]
    wv: np.ndarray  # [Hkv*d, Dm]
    wg: np.ndarray  # [Dm, 3*Hq]
    bg: np.ndarray  # [3*Hq]
    wo: np.ndarray  # [Dm, Hq*d]
    bq: Optional[np.ndarray] = None
    bk: Optional[np.ndarray] = None
    bv: Optional[np.ndarray] = None
    bo: Optional[np.ndarray] = None


@dataclass
class LayerForward:
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    gates: np.ndarray
    attn: ForwardResult
    y: np.ndarray


def layer_forward(orc: Oracle, x, w: LayerWeights, topk_idx=None) -> LayerForward:
    n = orc.N
    q = linear_forward(x, w.wq, w.bq).reshape(n, orc.Hq, orc.d)
    k = linear_forward(x, w.wk, w.bk).reshape(n, orc.Hkv, orc.d)
    v = linear_forward(x, w.wv, w.bv).reshape(n, orc.Hkv, orc.d)
    gates = gate_forward(x, w.wg, w.bg).reshape(n, orc.Hq, 3)
    attn = orc.forward(q, k, v, gates, topk_idx=topk_idx)
    y = linear_forward(attn.out.reshape(n, -1), w.wo, w.bo)
    return LayerForward(q, k, v, gates, attn, y)


def layer_backward(orc: Oracle, x, w: LayerWeights, f: LayerForward, dy) -> dict:
    """Gradients of sum(dy * y) w.r.t. x and every parameter; the selection f.attn.topk_idx is a constant."""
    n = orc.N
    do, dwo, dbo = linear_backward(f.attn.out.reshape(n, -1), w.wo, dy)
    b = orc.backward(f.q, f.k, f.v, f.gates, do.reshape(n, orc.Hq, orc.d), f.attn.topk_idx, out_branch=f.attn.out_branch)
    dxq, dwq, dbq = linear_backward(x, w.wq, b.dq.reshape(n, -1))
    dxk, dwk, dbk = linear_backward(x, w.wk, b.dk.reshape(n, -1))
    dxv, dwv, dbv = linear_backward(x, w.wv, b.dv.reshape(n, -1))
    dxg, dwg, dbg = gate_backward(x, w.wg, f.gates.reshape(n, -1), b.dgates.reshape(n, -1))
    return dict(dx=dxq + dxk + dxv + dxg, dwq=dwq, dwk=dwk, dwv=dwv, dwg=dwg, dbg=dbg, dwo=dwo, dbq=dbq, dbk=dbk,
                dbv=dbv, dbo=dbo, do=do, dq=b.dq, dk=b.dk, dv=b.dv, dgates=b.dgates)
