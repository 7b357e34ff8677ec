"""Comparison rules of the parity checks (test infrastructure, like the rest of this directory): the tolerances of
the floating-point outputs and the two-level contract for the selected sets.  Used by the tests and by the smoke run."""
from __future__ import annotations

import numpy as np

# spec tolerances: max-abs and mean-abs error, both relative to max|reference| of the tensor
TOL = {"bf16": (2e-2, 1e-3), "f32": (1e-5, 1e-5)}
# relative score margin inside which a selected block may legitimately differ from the fp64 oracle's choice
TOPK_MARGIN = {"bf16": 2e-3, "f32": 1e-5}


def rel_errors(got: np.ndarray, ref: np.ndarray):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = max(float(np.max(np.abs(ref))), 1e-30)
    diff = np.abs(got - ref)
    return float(diff.max() / den), float(diff.mean() / den)


def assert_close(got, ref, dtype: str, what: str, scale: float = 1.0):
    emax, emean = rel_errors(got, ref)
    tmax, tmean = TOL[dtype]
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), f"{what}: non-finite values"
    assert emax <= tmax * scale and emean <= tmean * scale, f"{what}: max {emax:.3e} (tol {tmax*scale:.1e}) mean {emean:.3e} (tol {tmean*scale:.1e})"
    return emax, emean


def check_topk(gpu_idx: np.ndarray, orc_fwd, orc, dtype: str, queries=None):
    """Two-level top-k contract: rows must equal the oracle's unless the differing blocks lie within the
    relative score margin of the T-th best score.  Returns the number of differing rows."""
    T = gpu_idx.shape[-1]
    rows = range(gpu_idx.shape[0]) if queries is None else queries
    b = orc.blocks
    eps = TOPK_MARGIN[dtype]
    differing = 0
    for t in rows:
        item = b.tok_item[t]
        s0, s1 = int(b.slc_batch[item]), int(b.slc_batch[item + 1])
        for g in range(gpu_idx.shape[1]):
            a, o = gpu_idx[t, g], orc_fwd.topk_idx[t, g]
            if np.array_equal(a, o):
                continue
            differing += 1
            av, ov = a[a >= 0], o[o >= 0]
            assert len(av) == len(ov) == min(T, s1 - s0), (t, g, a, o)
            assert np.all(np.diff(av) > 0) and av.min() >= s0 and av.max() < s1, (t, g, a)
            sc = orc_fwd.scores[t, g, : s1 - s0].astype(np.float64)
            kth = np.sort(sc)[::-1][len(ov) - 1]
            for blk in set(av.tolist()) ^ set(ov.tolist()):
                assert abs(sc[blk - s0] - kth) <= eps * kth, (t, g, blk, sc[blk - s0], kth)
    return differing


def check_block_arrays(arr: dict, n_tokens: int, n_batch: int) -> None:
    """Bounds of the index arrays a block handle exports (names of the binding's ARRAYS): every index that a kernel
    follows without a check of its own must stay inside the array it points into.  perm / inv_perm are inverse
    permutations of 0..N-1; the *_start arrays rise strictly from 0 to the size of what they cut (no empty block);
    the per-item ranges rise weakly (an item may be empty); tok_win names an existing window and is constant exactly
    on the window's own run of positions."""
    n = n_tokens
    perm, inv = arr["perm"].astype(np.int64), arr["inv_perm"].astype(np.int64)
    assert perm.shape == inv.shape == (n,)
    assert np.array_equal(np.sort(perm), np.arange(n)) and np.array_equal(inv[perm], np.arange(n))
    for name in ("cmp_start", "slc_start", "win_start"):
        s = arr[name].astype(np.int64)
        assert s[0] == 0 and s[-1] == n and np.all(np.diff(s) > 0), name
    nc, ns, nw = (len(arr[k]) - 1 for k in ("cmp_start", "slc_start", "win_start"))
    ch = arr["slc_child_start"].astype(np.int64)
    assert len(ch) == ns + 1 and ch[0] == 0 and ch[-1] == nc and np.all(np.diff(ch) > 0)
    for name, total in (("cmp_batch", nc), ("slc_batch", ns)):
        s = arr[name].astype(np.int64)
        assert len(s) == n_batch + 1 and s[0] == 0 and s[-1] == total and np.all(np.diff(s) >= 0), name
    tw = arr["tok_win"].astype(np.int64)
    assert tw.shape == (n,)
    if n:
        assert tw.min() >= 0 and tw.max() == nw - 1
        ws = arr["win_start"].astype(np.int64)
        assert np.array_equal(tw, np.repeat(np.arange(nw), np.diff(ws)))
