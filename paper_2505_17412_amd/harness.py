"""Plumbing shared by bench.py, the smoke run and the GPU tests: move a synthetic workload's arrays to the device, build
its block handle and run forward (+ backward) through the binding.  No arithmetic of the method lives here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import inputs


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
    from . import ssa
    return ssa.make_params(wl.n_tokens, wl.n_batch, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win, wl.topk, wl.n_heads_q,
                           wl.n_heads_kv, wl.head_dim, wl.dtype)


def build_blocks_gpu(wl: inputs.Workload):
    import torch
    from . import ssa
    p = params_of(wl)
    if wl.dims == 1:
        return p, ssa.ssa_build_blocks_1d(p, torch.from_numpy(wl.batch_offsets).cuda())
    coords = torch.from_numpy(wl.coords.reshape(-1, 3)).cuda() if wl.n_tokens else torch.zeros((1, 3), dtype=torch.int32, device="cuda")
    offs = torch.from_numpy(wl.batch_offsets).cuda()
    return p, ssa.ssa_build_blocks(p, coords, offs)


def run_gpu(wl: inputs.Workload, backward: bool = True, dout: Optional[np.ndarray] = None, blocks=None,
            idx_for_backward=None) -> GpuRun:
    """One forward (+ backward) of the workload through the C ABI; every output starts as NaN / a negative index so a
    value the library does not write shows up.  idx_for_backward: a function of the forward's index tensor (numpy
    int32 [N,Hkv,T]) returning the tensor the backward call is handed instead (Algorithm 1 takes I as an input)."""
    import torch
    from . import ssa
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
        if idx_for_backward is not None:
            idx = torch.from_numpy(np.ascontiguousarray(idx_for_backward(r.topk_idx), dtype=np.int32)).cuda()
        ssa.ssa_backward(p, blk, q, k, v, g, ob, lse, idx, do, dq, dk, dv, dg)
        torch.cuda.synchronize()
        r.dq, r.dk, r.dv, r.dgates = to_np(dq), to_np(dk), to_np(dv), to_np(dg)
    return r
