"""TEST INFRASTRUCTURE ONLY -- learned sparse 3D compression module in plain fp64 numpy.

Paper, Sec. "Sparse 3D Compression", eq. (5): a block-level token is delta(x + PE(x)) where PE is an absolute
positional encoding of the token's place inside its m_cmp^3 block and delta is a sparse 3D convolution followed by
a sparse 3D mean pool.  The paper gives no further detail; the readings fixed here:

  * PE is a table [m_cmp^3, C]; a token at (x, y, z) takes row ((x mod m)*m + (y mod m))*m + (z mod m);
  * the convolution is a 3x3x3 submanifold one over the whole sparse volume of the token's batch item: outputs
    exist at the active sites only, inactive neighbours contribute nothing, channels C -> C with a bias;
    weight[o] is [C_in, C_out] for offset o = ((dx+1)*3 + (dy+1))*3 + (dz+1), and the input taken is the token
    at coords + (dx, dy, dz);
  * the mean pool is over the active tokens of the compression block, as in the plain path;
  * coordinates are distinct inside an item (a duplicated site has no defined neighbourhood).

C = H_kv * d: the module mixes the channels of all KV heads.  Backward is the chain rule written out.
Nothing here is shared with, or imported by, the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

OFFSETS = [(dx, dy, dz) for dx in (-1, 0, 1) for dy in (-1, 0, 1) for dz in (-1, 0, 1)]  # index = the o above


def neighbor_table(coords: np.ndarray, batch_offsets: np.ndarray) -> np.ndarray:
    """int32 [N, 27]: caller index of the token at coords + OFFSETS[o] in the same item, or -1."""
    coords = np.asarray(coords, dtype=np.int64).reshape(-1, 3)
    offs = np.asarray(batch_offsets, dtype=np.int64)
    n = coords.shape[0]
    item = np.searchsorted(offs, np.arange(n), side="right") - 1
    where = {}
    for t in range(n):
        key = (int(item[t]), int(coords[t, 0]), int(coords[t, 1]), int(coords[t, 2]))
        assert key not in where, "coordinates must be distinct inside an item"
        where[key] = t
    nb = np.full((n, 27), -1, dtype=np.int32)
    for t in range(n):
        it, x, y, z = int(item[t]), int(coords[t, 0]), int(coords[t, 1]), int(coords[t, 2])
        for o, (dx, dy, dz) in enumerate(OFFSETS):
            nb[t, o] = where.get((it, x + dx, y + dy, z + dz), -1)
    return nb


def pe_index(coords: np.ndarray, m: int) -> np.ndarray:
    c = np.asarray(coords, dtype=np.int64).reshape(-1, 3) % m
    return ((c[:, 0] * m + c[:, 1]) * m + c[:, 2]).astype(np.int32)


@dataclass
class ModuleForward:
    u: np.ndarray    # [N, C] x + PE
    y: np.ndarray    # [N, C] convolution output
    x_cmp: np.ndarray  # [N_c, C] block means


@dataclass
class ModuleBackward:
    dx: np.ndarray     # [N, C]
    dpe: np.ndarray    # [m^3, C]
    dw: np.ndarray     # [27, C, C]
    dbias: np.ndarray  # [C]


class CompressionModule:
    """One tensor's (K's or V's) compression module on a fixed block structure."""

    def __init__(self, coords, batch_offsets, m_cmp: int, cmp_id: np.ndarray, n_cmp: int):
        self.nb = neighbor_table(coords, batch_offsets)
        self.pidx = pe_index(coords, m_cmp)
        self.cmp_id = np.asarray(cmp_id, dtype=np.int64)
        self.n_cmp = int(n_cmp)
        self.count = np.bincount(self.cmp_id, minlength=self.n_cmp).astype(np.float64)
        self.m = m_cmp

    def forward(self, x, pe, w, bias) -> ModuleForward:
        x = np.asarray(x, dtype=np.float64).reshape(x.shape[0], -1)
        pe = np.asarray(pe, dtype=np.float64).reshape(self.m ** 3, -1)
        w = np.asarray(w, dtype=np.float64)
        bias = np.asarray(bias, dtype=np.float64)
        u = x + pe[self.pidx]
        y = np.tile(bias, (x.shape[0], 1))
        for o in range(27):
            has = self.nb[:, o] >= 0
            y[has] += u[self.nb[has, o]] @ w[o]
        xc = np.zeros((self.n_cmp, x.shape[1]))
        np.add.at(xc, self.cmp_id, y)
        xc /= self.count[:, None]
        return ModuleForward(u, y, xc)

    def backward(self, x, pe, w, bias, dx_cmp) -> ModuleBackward:
        f = self.forward(x, pe, w, bias)
        w = np.asarray(w, dtype=np.float64)
        g = np.asarray(dx_cmp, dtype=np.float64).reshape(self.n_cmp, -1)
        dy = g[self.cmp_id] / self.count[self.cmp_id][:, None]
        dbias = dy.sum(axis=0)
        dw = np.zeros_like(w)
        du = np.zeros_like(f.u)
        for o in range(27):
            has = self.nb[:, o] >= 0
            src = self.nb[has, o]
            dw[o] = f.u[src].T @ dy[has]
            np.add.at(du, src, dy[has] @ w[o].T)
        dpe = np.zeros((self.m ** 3, du.shape[1]))
        np.add.at(dpe, self.pidx, du)
        return ModuleBackward(du, dpe, dw, dbias)
