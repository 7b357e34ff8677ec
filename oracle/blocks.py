"""TEST INFRASTRUCTURE ONLY -- plain numpy definition of the SSA block structure.

Paper, Sec. "Spatial Sparse Attention": space is cut into m^3 sub-grids and the active tokens of one
sub-grid form a block; tokens are sorted by block and the first-token index of each block (array C of
Algorithm 1) is kept.  Three granularities are used: compression (m_cmp), selection (m_slc), window (m_win).

Readings fixed here (the paper is silent on them):
  * a block's id is the rank of (batch item, Morton code of floor(coord / m)) among the non-empty blocks;
    Morton(x,y,z) interleaves bits as x -> bit 3i+2, y -> bit 3i+1, z -> bit 3i;
  * inside a block tokens are ordered by full-resolution Morton code, equal codes by caller index (stable);
  * block sides are powers of two, so one token order serves all three granularities.
This module is independent of the HIP library: it groups by explicit per-level keys and ``numpy.unique``;
it never shifts a sorted key to find a boundary.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict

import numpy as np


def morton3(x: np.ndarray, y: np.ndarray, z: np.ndarray, bits: int) -> np.ndarray:
    """Interleave the low ``bits`` bits of x, y, z (uint64 result): x highest, z lowest in each triple."""
    x = x.astype(np.uint64)
    y = y.astype(np.uint64)
    z = z.astype(np.uint64)
    code = np.zeros(x.shape, dtype=np.uint64)
    one = np.uint64(1)
    for i in range(bits):
        s = np.uint64(i)
        code |= ((x >> s) & one) << np.uint64(3 * i + 2)
        code |= ((y >> s) & one) << np.uint64(3 * i + 1)
        code |= ((z >> s) & one) << np.uint64(3 * i)
    return code


def _is_pow2(m: int) -> bool:
    return m >= 1 and (m & (m - 1)) == 0


@dataclass
class Blocks:
    n_tokens: int
    n_batch: int
    perm: np.ndarray  # int32 [N]  sorted position -> caller index
    inv_perm: np.ndarray  # int32 [N]  caller index -> sorted position
    tok_item: np.ndarray  # int32 [N]  caller order
    ids: Dict[str, np.ndarray]  # "cmp"/"slc"/"win" -> int32 [N] dense block id per token (caller order)
    n_blocks: Dict[str, int]
    start: Dict[str, np.ndarray]  # level -> int32 [n_blocks+1] first sorted position of each block
    cmp_parent: np.ndarray  # int32 [N_c] selection block of each compression block
    slc_child_start: np.ndarray  # int32 [N_s+1] compression-block range of each selection block
    cmp_batch: np.ndarray  # int32 [B+1]
    slc_batch: np.ndarray  # int32 [B+1]
    tok_win: np.ndarray  # int32 [N] window id of the token at each sorted position

    def members(self, level: str):
        """CSR (start, member caller-indices) of each block, members in sorted-position order."""
        return self.start[level], self.perm  # blocks are contiguous runs of the sorted order

    @property
    def s_max(self) -> int:
        return int(np.max(np.diff(self.slc_batch))) if self.n_batch else 0


def build_blocks(coords: np.ndarray, batch_offsets: np.ndarray, grid: int, m_cmp: int, m_slc: int,
                 m_win: int) -> Blocks:
    coords = np.asarray(coords, dtype=np.int64).reshape(-1, 3)
    offs = np.asarray(batch_offsets, dtype=np.int64)
    n = coords.shape[0]
    nb = offs.shape[0] - 1
    assert offs[0] == 0 and offs[-1] == n and np.all(np.diff(offs) >= 0)
    assert all(_is_pow2(m) for m in (m_cmp, m_slc, m_win)), "block sides must be powers of two"
    assert m_slc > m_cmp and m_slc % m_cmp == 0
    assert n == 0 or (coords.min() >= 0 and coords.max() < grid)
    bits = max(1, int(np.ceil(np.log2(max(grid, 2)))))
    item = (np.searchsorted(offs, np.arange(n), side="right") - 1).astype(np.int64)

    # token order: (item, full-resolution Morton code), stable
    code = morton3(coords[:, 0], coords[:, 1], coords[:, 2], bits)
    key = (item.astype(np.uint64) << np.uint64(3 * bits)) | code
    perm = np.argsort(key, kind="stable").astype(np.int32)
    inv_perm = np.empty(n, dtype=np.int32)
    inv_perm[perm] = np.arange(n, dtype=np.int32)

    ids: Dict[str, np.ndarray] = {}
    nblk: Dict[str, int] = {}
    start: Dict[str, np.ndarray] = {}
    blk_item: Dict[str, np.ndarray] = {}
    for level, m in (("cmp", m_cmp), ("slc", m_slc), ("win", m_win)):
        bc = coords // m
        bkey = (item.astype(np.uint64) << np.uint64(3 * bits)) | morton3(bc[:, 0], bc[:, 1], bc[:, 2], bits)
        uniq, inverse = np.unique(bkey, return_inverse=True)
        ids[level] = inverse.astype(np.int32)
        nblk[level] = int(uniq.shape[0])
        sorted_ids = ids[level][perm]
        assert np.all(np.diff(sorted_ids) >= 0), "blocks are not contiguous in the token order"
        start[level] = np.searchsorted(sorted_ids, np.arange(nblk[level] + 1), side="left").astype(np.int32)
        blk_item[level] = (uniq >> np.uint64(3 * bits)).astype(np.int64)

    # parent selection block of each compression block (any member token tells)
    cmp_parent = np.zeros(nblk["cmp"], dtype=np.int32)
    cmp_parent[ids["cmp"]] = ids["slc"]
    assert np.all(np.diff(cmp_parent) >= 0)
    slc_child_start = np.searchsorted(cmp_parent, np.arange(nblk["slc"] + 1), side="left").astype(np.int32)
    cmp_batch = np.searchsorted(blk_item["cmp"], np.arange(nb + 1), side="left").astype(np.int32)
    slc_batch = np.searchsorted(blk_item["slc"], np.arange(nb + 1), side="left").astype(np.int32)
    return Blocks(
        n_tokens=n, n_batch=nb, perm=perm, inv_perm=inv_perm, tok_item=item.astype(np.int32), ids=ids,
        n_blocks=nblk, start=start, cmp_parent=cmp_parent, slc_child_start=slc_child_start,
        cmp_batch=cmp_batch, slc_batch=slc_batch, tok_win=ids["win"][perm].astype(np.int32),
    )


def build_blocks_1d(batch_offsets: np.ndarray, l_cmp: int, l_slc: int, l_win: int) -> Blocks:
    """One-dimensional partition (the sequence-model blocks the paper's 3D partition takes the place of): item i is
    a sequence in the caller's order; a block is a run of l consecutive tokens counted from the start of its
    sequence, the last one possibly shorter.  Block ids count the blocks of all items in order."""
    offs = np.asarray(batch_offsets, dtype=np.int64)
    n = int(offs[-1])
    nb = offs.shape[0] - 1
    assert offs[0] == 0 and np.all(np.diff(offs) >= 0)
    assert l_slc > l_cmp and l_slc % l_cmp == 0 and l_win >= 1
    item = (np.searchsorted(offs, np.arange(n), side="right") - 1).astype(np.int64)
    pos = np.arange(n, dtype=np.int64) - offs[item]
    lens = np.diff(offs)
    ids: Dict[str, np.ndarray] = {}
    nblk: Dict[str, int] = {}
    start: Dict[str, np.ndarray] = {}
    per_item: Dict[str, np.ndarray] = {}
    for level, l in (("cmp", l_cmp), ("slc", l_slc), ("win", l_win)):
        cnt = -(-lens // l)  # blocks per item: ceil(len / l)
        first = np.concatenate([[0], np.cumsum(cnt)])
        per_item[level] = first
        ids[level] = (first[item] + pos // l).astype(np.int32)
        nblk[level] = int(first[-1])
        st = np.empty(nblk[level] + 1, dtype=np.int32)
        for it in range(nb):
            for j in range(int(cnt[it])):
                st[first[it] + j] = offs[it] + j * l
        st[-1] = n
        start[level] = st
    ratio = l_slc // l_cmp
    cmp_parent = np.empty(nblk["cmp"], dtype=np.int32)
    for it in range(nb):
        for j in range(int(per_item["cmp"][it + 1] - per_item["cmp"][it])):
            cmp_parent[per_item["cmp"][it] + j] = per_item["slc"][it] + j // ratio
    slc_child_start = np.searchsorted(cmp_parent, np.arange(nblk["slc"] + 1), side="left").astype(np.int32)
    ident = np.arange(n, dtype=np.int32)
    return Blocks(
        n_tokens=n, n_batch=nb, perm=ident, inv_perm=ident.copy(), tok_item=item.astype(np.int32), ids=ids,
        n_blocks=nblk, start=start, cmp_parent=cmp_parent, slc_child_start=slc_child_start,
        cmp_batch=per_item["cmp"].astype(np.int32), slc_batch=per_item["slc"].astype(np.int32),
        tok_win=ids["win"].astype(np.int32),
    )
