"""Helpers shared by the GPU parity tests: run the HIP path through the binding, compare with the oracle."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from paper_2505_17412_amd import inputs

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


@dataclass
class GpuRun:
    out: np.ndarray
    out_branch: np.ndarray
    lse: np.ndarray
    topk_idx: np.ndarray
    dq: Optional[np.ndarray] = None
    dk: Optional[np.ndarray] = None
    dv: Optional[np.ndarray] = None
    dgates: Optional[np.ndarray] = None


def to_dev(a: np.ndarray, dtype: str):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t.to(torch.float32)


def to_np(t) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def params_of(wl: inputs.Workload):
    from paper_2505_17412_amd import ssa
    return ssa.make_params(wl.n_tokens, wl.n_batch, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win, wl.topk, wl.n_heads_q,
                           wl.n_heads_kv, wl.head_dim, wl.dtype)


def build_blocks_gpu(wl: inputs.Workload):
    import torch
    from paper_2505_17412_amd import ssa
    p = params_of(wl)
    if wl.dims == 1:
        return p, ssa.ssa_build_blocks_1d(p, torch.from_numpy(wl.batch_offsets).cuda())
    coords = torch.from_numpy(wl.coords.reshape(-1, 3)).cuda() if wl.n_tokens else torch.zeros((1, 3), dtype=torch.int32, device="cuda")
    offs = torch.from_numpy(wl.batch_offsets).cuda()
    return p, ssa.ssa_build_blocks(p, coords, offs)


def run_gpu(wl: inputs.Workload, backward: bool = True, dout: Optional[np.ndarray] = None, blocks=None) -> GpuRun:
    import torch
    from paper_2505_17412_amd import ssa
    if blocks is None:
        p, blk = build_blocks_gpu(wl)
    else:
        p, blk = blocks
    n, hq, hkv, d, T = wl.n_tokens, wl.n_heads_q, wl.n_heads_kv, wl.head_dim, wl.topk
    td = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    q, k, v, g = (to_dev(a, wl.dtype) for a in (wl.q, wl.k, wl.v, wl.gates))
    out = torch.full((n, hq, d), float("nan"), dtype=td, device="cuda")
    ob = torch.full((3, n, hq, d), float("nan"), dtype=td, device="cuda")
    lse = torch.full((3, n, hq), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((n, hkv, T), -7, dtype=torch.int32, device="cuda")
    ssa.ssa_forward(p, blk, q, k, v, g, out, lse, idx, ob)
    torch.cuda.synchronize()
    r = GpuRun(to_np(out), to_np(ob), to_np(lse), to_np(idx))
    if backward:
        do = to_dev(wl.dout if dout is None else dout, wl.dtype)
        dq = torch.full_like(q, float("nan"))
        dk = torch.full_like(k, float("nan"))
        dv = torch.full_like(v, float("nan"))
        dg = torch.full_like(g, float("nan"))
        ssa.ssa_backward(p, blk, q, k, v, g, ob, lse, idx, do, dq, dk, dv, dg)
        torch.cuda.synchronize()
        r.dq, r.dk, r.dv, r.dgates = to_np(dq), to_np(dk), to_np(dv), to_np(dg)
    return r


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
