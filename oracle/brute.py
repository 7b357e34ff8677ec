"""TEST INFRASTRUCTURE ONLY -- brute-force SSA forward for tiny inputs, by a second, independent route.

Every branch is a dense N x N masked softmax (paper eq. (2)-(3)) with an explicit boolean mask built from a
dictionary-of-lists grouping of the voxel coordinates; nothing here uses sorted token orders, CSR arrays or
the C oracle.  Used only to pin ``ssa_oracle`` on inputs with a few dozen tokens.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np


def _morton_py(x: int, y: int, z: int, bits: int) -> int:
    code = 0
    for i in range(bits):
        code |= ((x >> i) & 1) << (3 * i + 2)
        code |= ((y >> i) & 1) << (3 * i + 1)
        code |= ((z >> i) & 1) << (3 * i)
    return code


def _masked_softmax_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: np.ndarray, scale: float):
    """q [N,d], k,v [M,d], mask [N,M] bool -> (o [N,d], lse [N], p [N,M])."""
    s = (q @ k.T) * scale
    s = np.where(mask, s, -np.inf)
    mx = s.max(axis=1, keepdims=True)
    e = np.exp(s - mx)
    den = e.sum(axis=1, keepdims=True)
    p = e / den
    return p @ v, (mx + np.log(den))[:, 0], p


def brute_forward(coords, batch_offsets, grid, m_cmp, m_slc, m_win, topk, q, k, v, gates, scale=None):
    coords = np.asarray(coords, dtype=np.int64)
    q, k, v, gates = (np.asarray(a, dtype=np.float64) for a in (q, k, v, gates))
    n, hq, d = q.shape
    hkv = k.shape[1]
    hs = hq // hkv
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    bits = max(1, int(np.ceil(np.log2(max(grid, 2)))))
    item = np.zeros(n, dtype=np.int64)
    for b in range(len(batch_offsets) - 1):
        item[batch_offsets[b]:batch_offsets[b + 1]] = b

    def group(m: int) -> Dict[Tuple[int, int, int, int], List[int]]:
        g: Dict[Tuple[int, int, int, int], List[int]] = {}
        for t in range(n):
            key = (int(item[t]), int(coords[t, 0] // m), int(coords[t, 1] // m), int(coords[t, 2] // m))
            g.setdefault(key, []).append(t)
        return g

    def ordered(g):  # block keys in id order: (item, Morton of the block coordinate)
        return sorted(g.keys(), key=lambda kk: (kk[0], _morton_py(kk[1], kk[2], kk[3], bits)))

    g_cmp, g_slc, g_win = group(m_cmp), group(m_slc), group(m_win)
    cmp_keys, slc_keys = ordered(g_cmp), ordered(g_slc)
    slc_index = {kk: i for i, kk in enumerate(slc_keys)}
    ratio = m_slc // m_cmp
    nc = len(cmp_keys)
    kc = np.stack([k[g_cmp[kk]].mean(axis=0) for kk in cmp_keys])  # [Nc,Hkv,d]
    vc = np.stack([v[g_cmp[kk]].mean(axis=0) for kk in cmp_keys])
    cmp_item = np.array([kk[0] for kk in cmp_keys])
    cmp_parent = np.array([slc_index[(kk[0], kk[1] // ratio, kk[2] // ratio, kk[3] // ratio)] for kk in cmp_keys])
    slc_item = np.array([kk[0] for kk in slc_keys])
    tok_slc = np.array([slc_index[(int(item[t]), *(int(c) // m_slc for c in coords[t]))] for t in range(n)])

    same_item_cmp = item[:, None] == cmp_item[None, :]  # [N,Nc]
    win_mask = np.zeros((n, n), dtype=bool)
    for members in g_win.values():
        for t in members:
            win_mask[t, members] = True

    out_b = np.zeros((3, n, hq, d))
    lse = np.zeros((3, n, hq))
    idx = np.full((n, hkv, topk), -1, dtype=np.int32)
    for g in range(hkv):
        score = np.zeros((n, len(slc_keys)))
        for hl in range(hs):
            h = g * hs + hl
            o, l, p = _masked_softmax_attention(q[:, h], kc[:, g], vc[:, g], same_item_cmp, scale)
            out_b[0, :, h], lse[0, :, h] = o, l
            for c in range(nc):
                score[:, cmp_parent[c]] += p[:, c]
        slc_mask = np.zeros((n, n), dtype=bool)
        score32 = score.astype(np.float32)
        for t in range(n):
            cand = [b for b in range(len(slc_keys)) if slc_item[b] == item[t]]
            best = sorted(cand, key=lambda b: (-float(score32[t, b]), b))[:topk]
            best = sorted(best)
            idx[t, g, :len(best)] = best
            slc_mask[t] = np.isin(tok_slc, best) & (item == item[t])
        for hl in range(hs):
            h = g * hs + hl
            out_b[1, :, h], lse[1, :, h], _ = _masked_softmax_attention(q[:, h], k[:, g], v[:, g], slc_mask, scale)
            out_b[2, :, h], lse[2, :, h], _ = _masked_softmax_attention(q[:, h], k[:, g], v[:, g], win_mask, scale)
    out = np.einsum("nhb,bnhd->nhd", gates, out_b)
    return dict(out=out, out_branch=out_b, lse=lse, topk_idx=idx, k_cmp=kc, v_cmp=vc)
