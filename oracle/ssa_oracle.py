"""TEST INFRASTRUCTURE ONLY -- Python face of the fp64 CPU oracle (``ssa_oracle.c`` + ``blocks.py``).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.  It never touches the HIP
library.  All arrays are in the caller's token order; see ``ssa_oracle.c`` for the definitions followed
(paper eq. (2)-(6), Algorithm 1, the window paragraph) and ``blocks.py`` for the block structure.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

from .blocks import Blocks, build_blocks, build_blocks_1d

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssa_oracle.c")
_LIB = os.path.join(_HERE, "libssa_oracle.so")


def build_library(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Problem(C.Structure):
    _fields_ = [
        ("N", C.c_int32), ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
        ("T", C.c_int32), ("Nc", C.c_int32), ("Ns", C.c_int32), ("Nw", C.c_int32), ("Smax", C.c_int32),
        ("scale", C.c_double),
        ("tok_item", C.c_void_p), ("cmp_id", C.c_void_p), ("slc_id", C.c_void_p), ("win_id", C.c_void_p),
        ("cmp_parent", C.c_void_p), ("cmp_item_start", C.c_void_p), ("slc_item_start", C.c_void_p),
        ("cmp_mem_start", C.c_void_p), ("cmp_mem", C.c_void_p),
        ("slc_mem_start", C.c_void_p), ("slc_mem", C.c_void_p),
        ("win_mem_start", C.c_void_p), ("win_mem", C.c_void_p),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        # SSA_ORACLE_LIB: another build of ssa_oracle.c to load instead (the sanitizer run of the pins uses it)
        _lib = C.CDLL(os.environ.get("SSA_ORACLE_LIB") or build_library())
        _lib.ssa_oracle_threads.restype = C.c_int
    return _lib


def n_threads() -> int:
    return int(_load().ssa_oracle_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


@dataclass
class ForwardResult:
    out: np.ndarray  # [N,Hq,d]
    out_branch: np.ndarray  # [3,N,Hq,d]
    lse: np.ndarray  # [3,N,Hq]
    topk_idx: np.ndarray  # int32 [N,Hkv,T], global selection-block ids ascending, -1 padded
    scores: Optional[np.ndarray]  # float32 [N,Hkv,Smax] or None
    k_cmp: np.ndarray  # [Nc,Hkv,d]
    v_cmp: np.ndarray


@dataclass
class BackwardResult:
    dq: np.ndarray
    dk: np.ndarray
    dv: np.ndarray
    dgates: np.ndarray
    dk_cmp: Optional[np.ndarray] = None  # only when block-level keys/values were supplied from outside
    dv_cmp: Optional[np.ndarray] = None


class Oracle:
    """SSA problem instance: block structure + hyper-parameters; forward/backward in fp64."""

    def __init__(self, coords, batch_offsets, grid, m_cmp, m_slc, m_win, topk, n_heads_q, n_heads_kv,
                 head_dim, scale: Optional[float] = None, blocks: Optional[Blocks] = None):
        assert n_heads_q % n_heads_kv == 0
        self.blocks = blocks if blocks is not None else build_blocks(coords, batch_offsets, grid, m_cmp, m_slc, m_win)
        b = self.blocks
        self.N, self.B = b.n_tokens, b.n_batch
        self.Hq, self.Hkv, self.d, self.T = n_heads_q, n_heads_kv, head_dim, topk
        self.scale = float(scale) if scale and scale > 0 else 1.0 / np.sqrt(head_dim)
        self._keep = dict(
            tok_item=_i32(b.tok_item), cmp_id=_i32(b.ids["cmp"]), slc_id=_i32(b.ids["slc"]),
            win_id=_i32(b.ids["win"]), cmp_parent=_i32(b.cmp_parent), cmp_item_start=_i32(b.cmp_batch),
            slc_item_start=_i32(b.slc_batch), cmp_mem_start=_i32(b.start["cmp"]), cmp_mem=_i32(b.perm),
            slc_mem_start=_i32(b.start["slc"]), slc_mem=_i32(b.perm), win_mem_start=_i32(b.start["win"]),
            win_mem=_i32(b.perm),
        )
        self.s_max = max(b.s_max, 1)
        self._prob = _Problem(
            N=self.N, B=self.B, Hq=self.Hq, Hkv=self.Hkv, d=self.d, T=self.T, Nc=b.n_blocks["cmp"],
            Ns=b.n_blocks["slc"], Nw=b.n_blocks["win"], Smax=self.s_max, scale=self.scale,
            **{k: v.ctypes.data for k, v in self._keep.items()},
        )

    # ----------------------------------------------------------------------------------------
    def pool(self, x: np.ndarray) -> np.ndarray:
        """Mean of x over the active tokens of each compression block (eq. (5), mean-pool part)."""
        x = _f64(x)
        xc = np.zeros((self.blocks.n_blocks["cmp"], self.Hkv, self.d), dtype=np.float64)
        _load().ssa_oracle_pool(C.byref(self._prob), _p(x), _p(xc))
        return xc

    def _qidx(self, queries) -> np.ndarray:
        return np.arange(self.N, dtype=np.int32) if queries is None else _i32(queries)

    def forward(self, q, k, v, gates, queries=None, topk_idx=None, want_scores: bool = False, k_cmp=None,
                v_cmp=None) -> ForwardResult:
        """Forward for ``queries`` (caller-order token indices; default all).  ``topk_idx`` given: use those
        selection sets instead of computing them.  ``k_cmp``/``v_cmp`` given: block-level keys/values from outside
        (e.g. the learned compression module) instead of the mean pool."""
        q, k, v, gates = _f64(q), _f64(k), _f64(v), _f64(gates)
        assert q.shape == (self.N, self.Hq, self.d) and k.shape == (self.N, self.Hkv, self.d)
        assert v.shape == k.shape and gates.shape == (self.N, self.Hq, 3)
        kc, vc = (self.pool(k), self.pool(v)) if k_cmp is None else (_f64(k_cmp), _f64(v_cmp))
        assert kc.shape == (self.blocks.n_blocks["cmp"], self.Hkv, self.d) and vc.shape == kc.shape
        qi = self._qidx(queries)
        out = np.zeros((self.N, self.Hq, self.d))
        ob = np.zeros((3, self.N, self.Hq, self.d))
        lse = np.zeros((3, self.N, self.Hq))
        idx = np.full((self.N, self.Hkv, self.T), -1, dtype=np.int32)
        sc = np.zeros((self.N, self.Hkv, self.s_max), dtype=np.float32) if want_scores else None
        iin = None if topk_idx is None else _i32(topk_idx)
        _load().ssa_oracle_forward(C.byref(self._prob), _p(q), _p(k), _p(v), _p(gates), _p(kc), _p(vc),
                                   C.c_int64(qi.shape[0]), _p(qi), _p(iin), _p(out), _p(ob), _p(lse), _p(sc), _p(idx))
        return ForwardResult(out, ob, lse, idx, sc, kc, vc)

    def backward(self, q, k, v, gates, dout, topk_idx, out_branch=None, queries=None, k_cmp=None, v_cmp=None):
        """Gradients of sum(dout * out) with the selection sets ``topk_idx`` held constant.  With ``k_cmp``/``v_cmp``
        (block-level keys/values from outside) the result also carries their gradients and dk, dv hold the selection
        and window branches only."""
        q, k, v, gates, dout = _f64(q), _f64(k), _f64(v), _f64(gates), _f64(dout)
        qi = self._qidx(queries)
        idx = _i32(topk_idx)
        if out_branch is None:
            out_branch = self.forward(q, k, v, gates, queries=qi, topk_idx=idx, k_cmp=k_cmp, v_cmp=v_cmp).out_branch
        ob = _f64(out_branch)
        given = k_cmp is not None
        kc, vc = (_f64(k_cmp), _f64(v_cmp)) if given else (self.pool(k), self.pool(v))
        dkc = np.zeros_like(kc) if given else None
        dvc = np.zeros_like(vc) if given else None
        dq = np.zeros((self.N, self.Hq, self.d))
        dk = np.zeros((self.N, self.Hkv, self.d))
        dv = np.zeros((self.N, self.Hkv, self.d))
        dg = np.zeros((self.N, self.Hq, 3))
        _load().ssa_oracle_backward(C.byref(self._prob), _p(q), _p(k), _p(v), _p(gates), _p(kc), _p(vc), _p(ob),
                                    _p(dout), C.c_int64(qi.shape[0]), _p(qi), _p(idx), _p(dq), _p(dk), _p(dv), _p(dg),
                                    _p(dkc), _p(dvc))
        res = BackwardResult(dq, dk, dv, dg)
        res.dk_cmp, res.dv_cmp = dkc, dvc
        return res

    def topk_from_scores(self, scores32: np.ndarray) -> np.ndarray:
        """Top-k decision alone on fp32 scores [N,Hkv,Smax] (column j = j-th selection block of the item)."""
        s = np.ascontiguousarray(scores32, dtype=np.float32)
        assert s.shape == (self.N, self.Hkv, self.s_max)
        b = self.blocks
        nv = np.repeat(np.diff(b.slc_batch)[b.tok_item], self.Hkv).astype(np.int32)
        base = np.repeat(b.slc_batch[:-1][b.tok_item], self.Hkv).astype(np.int32)
        out = np.full((self.N, self.Hkv, self.T), -1, dtype=np.int32)
        _load().ssa_oracle_topk(_p(s), C.c_int64(self.N * self.Hkv), C.c_int(self.s_max), C.c_int(self.T),
                                _p(nv), _p(base), _p(out))
        return out


def oracle_for(wl, **kw) -> Oracle:
    """Oracle for a ``paper_2505_17412_amd.inputs.Workload`` (voxel grid, or sequences when ``wl.dims == 1``)."""
    if getattr(wl, "dims", 3) == 1:
        kw = dict(kw, blocks=build_blocks_1d(wl.batch_offsets, wl.m_cmp, wl.m_slc, wl.m_win))
    return Oracle(wl.coords, wl.batch_offsets, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win, wl.topk,
                  wl.n_heads_q, wl.n_heads_kv, wl.head_dim, **kw)
