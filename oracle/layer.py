"""TEST INFRASTRUCTURE ONLY -- one full SSA attention layer in fp64: projections, gate predictor, attention, output
projection, chained from the oracles of the parts.

Paper: eq. (4) combines the three attention branches with gates "obtained by applying a linear layer followed by a
sigmoid activation to the input features"; queries, keys and values are linear projections of the same input features
and the result passes an output projection, as in any attention layer (Implementation Details: hidden dimension 1024,
grouped-query attention).  Reading: q = x Wq^T, k = x Wk^T, v = x Wv^T (optional biases), gates = sigmoid(x Wg + bg),
o = SSA(q, k, v, gates), y = o Wo^T (+ bo).  With the learned compression module (Sparse 3D Compression, eq. (5)) the
compression branch attends to delta(k + PE) and delta(v + PE), one module per tensor, instead of the mean pool.
Backward is the chain rule with the selected sets held constant.  Nothing here is shared with the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from .cmp_module import CompressionModule
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
    # learned compression module of the keys / of the values: positional table [m^3, C], weights [27, C, C], bias [C]
    pe_k: Optional[np.ndarray] = None
    wc_k: Optional[np.ndarray] = None
    bc_k: Optional[np.ndarray] = None
    pe_v: Optional[np.ndarray] = None
    wc_v: Optional[np.ndarray] = None
    bc_v: Optional[np.ndarray] = None


@dataclass
class LayerForward:
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    gates: np.ndarray
    attn: ForwardResult
    y: np.ndarray
    k_cmp: Optional[np.ndarray] = None  # [Nc, Hkv, d] block tokens of the learned module (None: mean pool)
    v_cmp: Optional[np.ndarray] = None


def block_tokens(orc: Oracle, module: CompressionModule, k, v, w: LayerWeights):
    n_c = orc.blocks.n_blocks["cmp"]
    kc = module.forward(k.reshape(orc.N, -1), w.pe_k, w.wc_k, w.bc_k).x_cmp.reshape(n_c, orc.Hkv, orc.d)
    vc = module.forward(v.reshape(orc.N, -1), w.pe_v, w.wc_v, w.bc_v).x_cmp.reshape(n_c, orc.Hkv, orc.d)
    return kc, vc


def layer_forward(orc: Oracle, x, w: LayerWeights, topk_idx=None, module: Optional[CompressionModule] = None) -> LayerForward:
    """``module`` (the block structure of the compression module) given: w must carry its six parameter arrays."""
    n = orc.N
    q = linear_forward(x, w.wq, w.bq).reshape(n, orc.Hq, orc.d)
    k = linear_forward(x, w.wk, w.bk).reshape(n, orc.Hkv, orc.d)
    v = linear_forward(x, w.wv, w.bv).reshape(n, orc.Hkv, orc.d)
    gates = gate_forward(x, w.wg, w.bg).reshape(n, orc.Hq, 3)
    kc, vc = block_tokens(orc, module, k, v, w) if module is not None else (None, None)
    attn = orc.forward(q, k, v, gates, topk_idx=topk_idx, k_cmp=kc, v_cmp=vc)
    y = linear_forward(attn.out.reshape(n, -1), w.wo, w.bo)
    return LayerForward(q, k, v, gates, attn, y, kc, vc)


def layer_backward(orc: Oracle, x, w: LayerWeights, f: LayerForward, dy, module: Optional[CompressionModule] = None) -> dict:
    """Gradients of sum(dy * y) w.r.t. x and every parameter; the selection f.attn.topk_idx is a constant.  With
    ``module``, f.k_cmp / f.v_cmp are the block tokens the attention saw and the gradients w.r.t. them flow back
    through the module onto dk and dv."""
    n = orc.N
    do, dwo, dbo = linear_backward(f.attn.out.reshape(n, -1), w.wo, dy)
    b = orc.backward(f.q, f.k, f.v, f.gates, do.reshape(n, orc.Hq, orc.d), f.attn.topk_idx, out_branch=f.attn.out_branch,
                     k_cmp=f.k_cmp if module is not None else None, v_cmp=f.v_cmp if module is not None else None)
    dk, dv = b.dk.reshape(n, -1), b.dv.reshape(n, -1)
    extra = {}
    if module is not None:
        mk = module.backward(f.k.reshape(n, -1), w.pe_k, w.wc_k, w.bc_k, b.dk_cmp)
        mv = module.backward(f.v.reshape(n, -1), w.pe_v, w.wc_v, w.bc_v, b.dv_cmp)
        dk, dv = dk + mk.dx, dv + mv.dx
        extra = dict(dpe_k=mk.dpe, dwc_k=mk.dw, dbc_k=mk.dbias, dpe_v=mv.dpe, dwc_v=mv.dw, dbc_v=mv.dbias,
                     dk_cmp=b.dk_cmp, dv_cmp=b.dv_cmp)
    dxq, dwq, dbq = linear_backward(x, w.wq, b.dq.reshape(n, -1))
    dxk, dwk, dbk = linear_backward(x, w.wk, dk)
    dxv, dwv, dbv = linear_backward(x, w.wv, dv)
    dxg, dwg, dbg = gate_backward(x, w.wg, f.gates.reshape(n, -1), b.dgates.reshape(n, -1))
    return dict(dx=dxq + dxk + dxv + dxg, dwq=dwq, dwk=dwk, dwv=dwv, dwg=dwg, dbg=dbg, dwo=dwo, dbq=dbq, dbk=dbk,
                dbv=dbv, dbo=dbo, do=do, dq=b.dq, dk=dk.reshape(n, orc.Hkv, orc.d), dv=dv.reshape(n, orc.Hkv, orc.d),
                dgates=b.dgates, **extra)
