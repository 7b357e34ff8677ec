"""SSA forward+backward throughput on one MI355X (config: ~60k-token shell on a 128^3 grid).

Prints ONE JSON line: whole-step tokens/s, the roofline position of the dominant kernel (live HIP-event timing
through the library's profiling hook) and the fp64 CPU oracle timed on a bounded query sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector ALU
# kernels of ssa_forward as the profiling hook names them (prep_sort_pool also runs in ssa_backward)
FWD_KERNELS = ("prep_sort_pool", "cmp_fwd_scores_topk", "fwd_invert_selection", "slc_fwd", "win_fwd", "slc_merge_combine")
HBM_PEAK_GBS = 8000.0


def algorithmic_flops(wl, blk_arrays, idx):
    """Pair counts from the run's real block structure and selected sets (never dense N^2)."""
    import numpy as np
    d, hq, hkv = wl.head_dim, wl.n_heads_q, wl.n_heads_kv
    hs = hq // hkv
    perm, tok_win, win_start = blk_arrays["perm"], blk_arrays["tok_win"], blk_arrays["win_start"]
    cmp_batch, slc_start = blk_arrays["cmp_batch"], blk_arrays["slc_start"]
    n_item = np.diff(wl.batch_offsets.astype(np.int64))
    pairs_cmp = int(np.sum(n_item * np.diff(cmp_batch.astype(np.int64)))) * hq
    win_len = np.diff(win_start.astype(np.int64))
    pairs_win = int(np.sum(win_len[tok_win])) * hq
    blk_len = np.concatenate([np.diff(slc_start.astype(np.int64)), [0]])  # index -1 -> 0
    pairs_slc = int(np.sum(blk_len[idx])) * hs
    return dict(cmp=pairs_cmp, slc=pairs_slc, win=pairs_win, d=d)


# bench.py kernel name -> kernel name prefix in the rocprofv3 summaries
ROCPROF_NAME = {
    "cmp_fwd_scores_topk": "m_cmp_fwd<", "slc_fwd": "m_slc_fwd_bc<", "win_fwd": "m_win_fwd<",
    "bwd_dq_cmp_win": "m_bwd_dq<{d},", "bwd_dq_slc": "m_bwd_dq_bc<{d},",
    "bwd_dkv_win": "m_bwd_dkv<{d}, {kb}, 0,", "bwd_dkv_slc": "m_bwd_dkv<{d}, {kb}, 1,", "bwd_dkv_cmp": "m_bwd_dkv<{d}, {kb}, 2,",
}


def kernel_source_hash():
    """sha256 over the library's sources (kernels and headers): a profile summary names the hash of the sources it was
    measured on, so a figure read from it is only reported while the sources are still those."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2505_17412_amd", "csrc")
    files = sorted(os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith((".hip", ".h")))
    for f in files + [os.path.join(ROOT, "include", "ssa.h")]:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(kernel, workload, d):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 FETCH_SIZE/WRITE_SIZE summary of this workload
    (scaled columns, MiB) with the summary it came from, or (None, None) when no summary covers the kernel or the
    summary was measured on other sources than the ones in the tree."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}_fwd_bwd.md")
    pat = ROCPROF_NAME.get(kernel)
    if pat is None or not os.path.exists(path):
        return None, None
    pat = pat.format(d=d, kb=1 if d >= 128 else 2)
    text = open(path).read()
    src = kernel_source_hash()
    if f"kernel sources sha256/16: {src}" not in text:
        return None, None
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 5 and cells[0].startswith(pat):
            return int((float(cells[3]) + float(cells[4])) * 1024 * 1024), {"summary": os.path.relpath(path, ROOT), "kernel_sources": src}
    return None, None


def _imports():
    import torch
    from paper_2505_17412_amd import harness as util, inputs, ssa
    return torch, inputs, ssa, util


def kernel_times(wl, steps):
    """Average HIP-event time per kernel (ms) over `steps` forward+backward passes; also returns what the work count
    needs: the handle's arrays and the selected sets."""
    torch, _, ssa, util = _imports()
    n, hq, hkv, T = wl.n_tokens, wl.n_heads_q, wl.n_heads_kv, wl.topk
    p, blk = util.build_blocks_gpu(wl)
    q, k, v, g, do = (util.to_dev(a, wl.dtype) for a in (wl.q, wl.k, wl.v, wl.gates, wl.dout))
    out = torch.empty_like(q)
    ob = torch.empty((3,) + tuple(q.shape), dtype=q.dtype, device="cuda")
    lse = torch.empty((3, n, hq), dtype=torch.float32, device="cuda")
    idx = torch.empty((n, hkv, T), dtype=torch.int32, device="cuda")
    dq, dk, dv, dg = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v), torch.empty_like(g)
    wsf = torch.empty(ssa.ssa_workspace_bytes(p, blk, False), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(ssa.ssa_workspace_bytes(p, blk, True), dtype=torch.uint8, device="cuda")

    def step():
        ssa.ssa_forward(p, blk, q, k, v, g, out, lse, idx, ob, wsf)
        ssa.ssa_backward(p, blk, q, k, v, g, ob, lse, idx, do, dq, dk, dv, dg, wsb)

    step()
    torch.cuda.synchronize()
    ssa.ssa_profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    prof = ssa.ssa_profile_get()
    ssa.ssa_profile_enable(False)
    arrays = {nm: blk.export(nm).cpu().numpy() for nm in ("perm", "tok_win", "win_start", "cmp_batch", "slc_start")}
    sel = idx.cpu().numpy()
    blk.destroy()
    return {nm: tot / cnt for nm, (tot, cnt) in prof.items()}, arrays, sel


def dense_dq_ms(kd, pairs):
    """Window share of the dQ kernel that handles the compression and window branches (split by their pair counts): in the
    dense stand-in the window is the whole item, the compression branch a few per cent of it."""
    return kd["bwd_dq_cmp_win"] * pairs["win"] / max(pairs["win"] + pairs["cmp"], 1)


# Token sweep of the sparse path against dense attention computed by the same library (the window branch with one
# window over the whole grid is plain dense variable-length attention).  Shells of the bench workload's recipe at
# three grid sizes: (grid, size factor f, half-width w).
SWEEP_POINTS = [(32, 0.55, 1.0), (64, 0.45, 1.0), (64, 0.55, 1.5), (128, 0.55, 0.75), (128, 0.55, 1.5), (128, 0.55, 3.0)]


def dense_sweep(args):
    """One JSON line per sweep point: per-kernel HIP-event times of the sparse configuration (m = 4/8/8, top-k 16)
    and of the dense stand-in (m_win = grid, top-k 1: the window kernels then visit every (query, key) pair)."""
    import torch
    from paper_2505_17412_amd import harness as util, inputs, ssa

    torch.cuda.set_device(0)

    fwd_names = FWD_KERNELS
    for grid, f, w in SWEEP_POINTS:
        sparse = inputs.make_workload("g128", grid=grid, f=f, w=w)
        dense = inputs.make_workload("g128", grid=grid, f=f, w=w, m=(4, 8, grid), topk=1)
        n = sparse.n_tokens
        ks = kernel_times(sparse, 3)[0]
        kd, d_arrays, d_sel = kernel_times(dense, 2 if n > 50000 else 3)
        dense_pairs = algorithmic_flops(dense, d_arrays, d_sel)
        # prep_sort_pool runs once in forward and once in backward; its average is booked on both sides
        s_fwd = sum(ks.get(nm, 0.0) for nm in fwd_names)
        s_bwd = sum(v_ for nm, v_ in ks.items() if nm not in fwd_names) + ks["prep_sort_pool"]
        d_fwd = kd["win_fwd"]
        d_bwd = dense_dq_ms(kd, dense_pairs) + kd["bwd_dkv_win"] + kd["bwd_pre_delta"]
        line = {"sweep": "ssa_vs_dense", "grid": grid, "n_tokens": n, "heads": [sparse.n_heads_q, sparse.n_heads_kv],
                "head_dim": sparse.head_dim, "ssa_fwd_ms": round(s_fwd, 3), "ssa_bwd_ms": round(s_bwd, 3),
                "dense_fwd_ms": round(d_fwd, 3), "dense_bwd_ms": round(d_bwd, 3),
                "speedup_fwd": round(d_fwd / s_fwd, 2), "speedup_bwd": round(d_bwd / s_bwd, 2),
                "speedup_fwd_bwd": round((d_fwd + d_bwd) / (s_fwd + s_bwd), 2),
                "dense_fwd_tflops": round(4 * sparse.head_dim * n * n * sparse.n_heads_q / (d_fwd * 1e-3) / 1e12, 1)}
        print(json.dumps(line), flush=True)





def seq1d_bench(args):
    """One JSON line per sequence workload: the same kernels on the one-dimensional partition of sequence models
    (compression blocks of 32 tokens, selection blocks of 64, windows of 512, top-16), against dense attention over
    the same sequences (one window per sequence)."""
    torch, inputs, ssa, util = _imports()
    torch.cuda.set_device(0)
    for lens in ((65536,), (16384,) * 4):
        n = sum(lens)
        sparse = inputs.make_sequence_workload(2001, lens)
        dense = inputs.make_sequence_workload(2001, lens, l=(32, 64, max(lens)), topk=1)
        ks, arrays, sel = kernel_times(sparse, 3)
        kd, d_arrays, d_sel = kernel_times(dense, 2)
        dense_pairs = algorithmic_flops(dense, d_arrays, d_sel)
        pairs = algorithmic_flops(sparse, arrays, sel)
        total_pairs = pairs["cmp"] + pairs["slc"] + pairs["win"]
        s_fwd = sum(ks.get(nm, 0.0) for nm in FWD_KERNELS)
        s_bwd = sum(v_ for nm, v_ in ks.items() if nm not in FWD_KERNELS) + ks["prep_sort_pool"]
        d_fwd = kd["win_fwd"]
        d_bwd = dense_dq_ms(kd, dense_pairs) + kd["bwd_dkv_win"] + kd["bwd_pre_delta"]
        flops = 14 * sparse.head_dim * total_pairs
        line = {"bench": "sequence_partition", "lens": list(lens), "n_tokens": n, "blocks": [32, 64, 512], "topk": 16,
                "heads": [sparse.n_heads_q, sparse.n_heads_kv], "head_dim": sparse.head_dim,
                "ssa_fwd_ms": round(s_fwd, 3), "ssa_bwd_ms": round(s_bwd, 3),
                "tokens_per_s": round(n / ((s_fwd + s_bwd) * 1e-3)),
                "pairs_cmp_slc_win": [pairs["cmp"], pairs["slc"], pairs["win"]],
                "algorithmic_tflops": round(flops / ((s_fwd + s_bwd) * 1e-3) / 1e12, 1),
                "frac_of_mfma_peak": round(flops / ((s_fwd + s_bwd) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "dense_fwd_ms": round(d_fwd, 3), "dense_bwd_ms": round(d_bwd, 3),
                "speedup_fwd_bwd": round((d_fwd + d_bwd) / (s_fwd + s_bwd), 2),
                "kernel_ms": {k_: round(v_, 3) for k_, v_ in ks.items()}}
        print(json.dumps(line), flush=True)


def cmp_module_bench(args):
    """One JSON line: the learned compression module (eq. (5)) at the benchmark workload, alone and inside a full
    training step (two modules forward, attention with their block-level tokens, everything backward)."""
    import numpy as np
    import torch
    from paper_2505_17412_amd import harness as util, inputs, ssa

    torch.cuda.set_device(0)
    wl = inputs.make_workload(args.workload)
    n, hq, hkv, d, T = wl.n_tokens, wl.n_heads_q, wl.n_heads_kv, wl.head_dim, wl.topk
    c, m3 = hkv * d, wl.m_cmp ** 3
    p, blk = util.build_blocks_gpu(wl)
    nc = blk.counts()[0]
    q, k, v, g, do = (util.to_dev(a, wl.dtype) for a in (wl.q, wl.k, wl.v, wl.gates, wl.dout))
    gen = torch.Generator(device="cuda").manual_seed(7)
    rand = lambda *shape: torch.randn(shape, generator=gen, device="cuda")
    wts = [((0.5 * rand(m3, c)).bfloat16(), (rand(27, c, c) / (9.0 * c) ** 0.5).bfloat16(), (0.1 * rand(c)).bfloat16())
           for _ in range(2)]
    kc, vc = (torch.empty((nc, hkv, d), dtype=torch.bfloat16, device="cuda") for _ in range(2))
    out = torch.empty_like(q)
    ob = torch.empty((3,) + tuple(q.shape), dtype=q.dtype, device="cuda")
    lse = torch.empty((3, n, hq), dtype=torch.float32, device="cuda")
    idx = torch.empty((n, hkv, T), dtype=torch.int32, device="cuda")
    dq, dk, dv, dg = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v), torch.empty_like(g)
    dkc, dvc = (torch.empty((nc, hkv, d), dtype=torch.float32, device="cuda") for _ in range(2))
    grads = [(torch.empty((m3, c), device="cuda"), torch.empty((27, c, c), device="cuda"), torch.empty((c,), device="cuda"))
             for _ in range(2)]
    wsf = torch.empty(ssa.ssa_workspace_bytes(p, blk, False), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(ssa.ssa_workspace_bytes(p, blk, True), dtype=torch.uint8, device="cuda")
    wmf = torch.empty(ssa.ssa_compress_workspace_bytes(p, blk, False), dtype=torch.uint8, device="cuda")
    wmb = torch.empty(ssa.ssa_compress_workspace_bytes(p, blk, True), dtype=torch.uint8, device="cuda")

    def step():
        ssa.ssa_compress_forward(p, blk, k, *wts[0], kc, wmf)
        ssa.ssa_compress_forward(p, blk, v, *wts[1], vc, wmf)
        ssa.ssa_forward_pooled(p, blk, q, k, v, g, kc, vc, out, lse, idx, ob, wsf)
        ssa.ssa_backward_pooled(p, blk, q, k, v, g, kc, vc, ob, lse, idx, do, dq, dk, dv, dg, dkc, dvc, wsb)
        ssa.ssa_compress_backward(p, blk, k, *wts[0], dkc, dk, *grads[0], wmb)
        ssa.ssa_compress_backward(p, blk, v, *wts[1], dvc, dv, *grads[1], wmb)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    ssa.ssa_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = {nm: tot / cnt for nm, (tot, cnt) in ssa.ssa_profile_get().items()}
    ssa.ssa_profile_enable(False)
    # (token, offset) pairs with an active neighbour, counted from the coordinates (single item)
    co = wl.coords.astype(np.int64)
    code = (co[:, 0] * 4096 + co[:, 1]) * 4096 + co[:, 2]
    srt = np.sort(code)
    pairs = 0
    for dx in (-1, 0, 1):
        for dy in (-1, 0, 1):
            for dz in (-1, 0, 1):
                cc = co + np.array([dx, dy, dz])
                ok = np.all((cc >= 0) & (cc < wl.grid), axis=1)
                want = (cc[:, 0] * 4096 + cc[:, 1]) * 4096 + cc[:, 2]
                j = np.clip(np.searchsorted(srt, want), 0, n - 1)
                pairs += int(np.sum(ok & (srt[j] == want)))
    flop_fwd = 2.0 * c * c * pairs
    line = {"bench": "learned_compression_module", "workload": args.workload, "n_tokens": n, "channels": c,
            "neighbour_pairs": pairs, "module_fwd_ms_per_tensor": round(prof["cmp_module_fwd"], 4),
            "module_bwd_ms_per_tensor": round(prof["cmp_module_bwd"], 4),
            "module_fwd_algorithmic_tflops": round(flop_fwd / (prof["cmp_module_fwd"] * 1e-3) / 1e12, 2),
            "module_bwd_algorithmic_tflops": round(2 * flop_fwd / (prof["cmp_module_bwd"] * 1e-3) / 1e12, 2),
            "step_with_modules_ms": round(ms, 4), "tokens_per_s_with_modules": round(n / (ms * 1e-3), 1),
            "steps": args.steps, "warmup": args.warmup}
    print(json.dumps(line), flush=True)


def gate_bench(args):
    """One JSON line: the gate predictor (sigmoid of a linear layer d_model -> 3*Hq) at the benchmark workload's token
    count, against the HBM roofline (it streams x once forward; x once and dx twice backward)."""
    import torch
    from paper_2505_17412_amd import inputs, ssa

    torch.cuda.set_device(0)
    wl = inputs.make_workload(args.workload, with_tensors=False)
    n, hq = wl.n_tokens, wl.n_heads_q
    dm, j = hq * wl.head_dim, 3 * hq
    p = ssa.make_params(n, 1, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win, wl.topk, hq, wl.n_heads_kv, wl.head_dim, "bf16")
    gen = torch.Generator(device="cuda").manual_seed(11)
    x = torch.randn((n, dm), generator=gen, device="cuda").bfloat16()
    w = (torch.randn((dm, j), generator=gen, device="cuda") / dm ** 0.5).bfloat16()
    b = torch.randn((j,), generator=gen, device="cuda").bfloat16()
    dg = torch.randn((n, hq, 3), generator=gen, device="cuda").bfloat16()
    gates = torch.empty((n, hq, 3), dtype=torch.bfloat16, device="cuda")
    dx = torch.zeros_like(x)
    dw = torch.empty((dm, j), device="cuda")
    db = torch.empty((j,), device="cuda")
    wsf = torch.empty(ssa.ssa_gate_workspace_bytes(p, dm, False), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(ssa.ssa_gate_workspace_bytes(p, dm, True), dtype=torch.uint8, device="cuda")

    def step():
        ssa.ssa_gate_forward(p, dm, x, w, b, gates, wsf)
        ssa.ssa_gate_backward(p, dm, x, w, gates, dg, dx, dw, db, wsb)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ssa.ssa_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = {nm: tot / cnt for nm, (tot, cnt) in ssa.ssa_profile_get().items()}
    ssa.ssa_profile_enable(False)
    fwd_bytes = n * dm * 2 + n * j * 2
    bwd_bytes = n * dm * 2 + 2 * n * dm * 2 + 2 * n * j * 2
    line = {"bench": "gate_predictor", "workload": args.workload, "n_tokens": n, "d_model": dm, "gates_per_token": j,
            "fwd_ms": round(prof["gate_fwd"], 4), "bwd_ms": round(prof["gate_bwd"], 4),
            "fwd_algorithmic_gbps": round(fwd_bytes / (prof["gate_fwd"] * 1e-3) / 1e9, 1),
            "bwd_algorithmic_gbps": round(bwd_bytes / (prof["gate_bwd"] * 1e-3) / 1e9, 1),
            "hbm_peak_gbps": HBM_PEAK_GBS, "steps": args.steps, "warmup": args.warmup}
    print(json.dumps(line), flush=True)


def linear_bench(args):
    """One JSON line per projection shape of the layer (hidden -> Hq*d and hidden -> Hkv*d) at the benchmark workload's
    token count, against the bf16 MFMA roofline: 2*N*d_in*d_out FLOPs forward, twice that backward (dx and dW)."""
    import torch
    from paper_2505_17412_amd import inputs, ssa

    torch.cuda.set_device(0)
    wl = inputs.make_workload(args.workload, with_tensors=False)
    n = wl.n_tokens
    dm = wl.n_heads_q * wl.head_dim
    gen = torch.Generator(device="cuda").manual_seed(13)
    for d_in, d_out in ((dm, dm), (dm, wl.n_heads_kv * wl.head_dim)):
        x = torch.randn((n, d_in), generator=gen, device="cuda").bfloat16()
        w = (torch.randn((d_out, d_in), generator=gen, device="cuda") / d_in ** 0.5).bfloat16()
        b = torch.randn((d_out,), generator=gen, device="cuda").bfloat16()
        dy = torch.randn((n, d_out), generator=gen, device="cuda").bfloat16()
        y = torch.empty((n, d_out), dtype=torch.bfloat16, device="cuda")
        dx = torch.empty_like(x)
        dw = torch.empty((d_out, d_in), device="cuda")
        db = torch.empty((d_out,), device="cuda")
        ws = torch.empty(ssa.ssa_linear_workspace_bytes(n, d_in, d_out, True), dtype=torch.uint8, device="cuda")

        def step():
            ssa.ssa_linear_forward(x, w, b, y)
            ssa.ssa_linear_backward(x, w, dy, dx, dw, db, ws)

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        ssa.ssa_profile_enable(True)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        prof = {nm: tot / cnt for nm, (tot, cnt) in ssa.ssa_profile_get().items()}
        ssa.ssa_profile_enable(False)
        flops = 2.0 * n * d_in * d_out
        line = {"bench": "linear_projection", "workload": args.workload, "n_tokens": n, "d_in": d_in, "d_out": d_out,
                "fwd_ms": round(prof["linear_fwd"], 4), "bwd_ms": round(prof["linear_bwd"], 4),
                "fwd_tflops": round(flops / (prof["linear_fwd"] * 1e-3) / 1e12, 1),
                "bwd_tflops": round(2 * flops / (prof["linear_bwd"] * 1e-3) / 1e12, 1),
                "fwd_frac_of_mfma_peak": round(flops / (prof["linear_fwd"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "bwd_frac_of_mfma_peak": round(2 * flops / (prof["linear_bwd"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "steps": args.steps, "warmup": args.warmup}
        print(json.dumps(line), flush=True)


def layer_bench(args):
    """One JSON line: a full SSA attention layer (q/k/v projections, gate predictor, attention, output projection;
    hidden dimension = Hq * d) forward + backward at the benchmark workload, timed as a whole with events on the
    stream, plus the per-part totals from the library's profiling hook."""
    import torch
    from paper_2505_17412_amd import harness as util, inputs, ssa

    torch.cuda.set_device(0)
    wl = inputs.make_workload(args.workload, with_tensors=False)
    n, hq, hkv, d = wl.n_tokens, wl.n_heads_q, wl.n_heads_kv, wl.head_dim
    dm, cq, ckv = hq * d, hq * d, hkv * d
    p, blk = util.build_blocks_gpu(wl)
    gen = torch.Generator(device="cuda").manual_seed(17)
    rnd = lambda *s_, scale=1.0: (torch.randn(s_, generator=gen, device="cuda") * scale).bfloat16()
    x, dy = rnd(n, dm), rnd(n, dm)
    w = dict(wq=rnd(cq, dm, scale=dm ** -0.5), wk=rnd(ckv, dm, scale=dm ** -0.5), wv=rnd(ckv, dm, scale=dm ** -0.5),
             wg=rnd(dm, 3 * hq, scale=dm ** -0.5), bg=rnd(3 * hq), wo=rnd(dm, cq, scale=cq ** -0.5))
    if args.learned_cmp:  # the learned compression module on keys and values instead of the mean pool
        for t in ("k", "v"):
            w["pe_" + t] = rnd(wl.m_cmp ** 3, ckv, scale=0.5)
            w["wc_" + t] = rnd(27, ckv, ckv, scale=(9.0 * ckv) ** -0.5)
            w["bc_" + t] = rnd(ckv, scale=0.1)
    grads = {"d" + k_: torch.empty(v_.shape, device="cuda") for k_, v_ in w.items()}
    y, dx = torch.empty_like(x), torch.empty_like(x)
    saved = torch.empty(ssa.ssa_layer_saved_bytes(p)[0], dtype=torch.uint8, device="cuda")
    wsf = torch.empty(ssa.ssa_layer_workspace_bytes(p, blk, dm, False), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(ssa.ssa_layer_workspace_bytes(p, blk, dm, True), dtype=torch.uint8, device="cuda")

    def step():
        ssa.ssa_layer_forward(p, blk, x, w, y, saved, wsf)
        ssa.ssa_layer_backward(p, blk, x, w, saved, dy, dx, grads, wsb)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    ssa.ssa_profile_enable(True)
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    prof = {nm: tot / 3 for nm, (tot, cnt) in ssa.ssa_profile_get().items()}
    ssa.ssa_profile_enable(False)
    lin = prof.get("linear_fwd", 0.0) + prof.get("linear_bwd", 0.0)
    gate = prof.get("gate_fwd", 0.0) + prof.get("gate_bwd", 0.0)
    module = sum(v_ for k_, v_ in prof.items() if k_.startswith("cmp_module"))
    attn = sum(v_ for k_, v_ in prof.items() if not k_.startswith(("linear", "gate", "cmp_module")))
    gemm_flops = 6.0 * n * dm * (2 * cq + 2 * ckv)  # forward 2 + backward 4 FLOPs per (token, weight)
    line = {"bench": "ssa_layer", "workload": args.workload, "n_tokens": n, "d_model": dm, "heads": [hq, hkv], "head_dim": d,
            "ms_per_layer_step": round(ms, 3), "tokens_per_s": round(n / (ms * 1e-3)),
            "compression": "learned module" if args.learned_cmp else "mean pool",
            "part_ms": {"projections": round(lin, 3), "gate_predictor": round(gate, 3), "attention": round(attn, 3),
                        "compression_module": round(module, 3)},
            "projection_tflops": round(gemm_flops / (lin * 1e-3) / 1e12, 1) if lin > 0 else None,
            "saved_activation_mib": round(saved.numel() / 2 ** 20, 1), "steps": args.steps, "warmup": args.warmup}
    print(json.dumps(line), flush=True)


def ablation_sweep(args):
    """Stress workload (thick shell, ~150k tokens, head_dim 128): top-k in {8, 16, 32} x window side in {4, 8}, one
    JSON line each with every branch's forward+backward time and its algorithmic TFLOP/s against the MFMA peak."""
    torch, inputs, ssa, util = _imports()
    torch.cuda.set_device(0)
    for topk in (8, 16, 32):
        for m_win in (4, 8):
            wl = inputs.make_workload("g128_thick", topk=topk, m=(4, 8, m_win))
            n, d = wl.n_tokens, wl.head_dim
            ks, arrays, sel = kernel_times(wl, 2)
            pairs = algorithmic_flops(wl, arrays, sel)
            # the compression and window branches share a dQ launch: its time is split by their pair counts
            dq_cw = ks["bwd_dq_cmp_win"]
            f_c = pairs["cmp"] / max(pairs["cmp"] + pairs["win"], 1)
            branch_ms = {
                "cmp": ks["cmp_fwd_scores_topk"] + dq_cw * f_c + ks["bwd_dkv_cmp"],
                "slc": ks["slc_fwd"] + ks["fwd_invert_selection"] + ks["slc_merge_combine"] + ks["bwd_dq_slc"] + ks["bwd_dq_merge"]
                       + ks["bwd_dkv_slc"] + ks["bwd_invert_selection"],
                "win": ks["win_fwd"] + dq_cw * (1 - f_c) + ks["bwd_dkv_win"],
            }
            other = sum(ks.values()) + ks["prep_sort_pool"] - sum(branch_ms.values())
            total = sum(branch_ms.values()) + other
            tf = {b: 14 * d * pairs[b] / (branch_ms[b] * 1e-3) / 1e12 for b in branch_ms}
            line = {"bench": "stress_ablation", "workload": "g128_thick", "n_tokens": n, "head_dim": d,
                    "heads": [wl.n_heads_q, wl.n_heads_kv], "topk": topk, "m_win": m_win,
                    "fwd_bwd_ms": round(total, 3), "tokens_per_s": round(n / (total * 1e-3)),
                    "branch_ms": {b: round(v_, 3) for b, v_ in branch_ms.items()}, "other_ms": round(other, 3),
                    "branch_tflops": {b: round(v_, 1) for b, v_ in tf.items()},
                    "branch_frac_of_mfma_peak": {b: round(v_ / MFMA_BF16_PEAK_TFLOPS, 4) for b, v_ in tf.items()},
                    "whole_step_frac_of_mfma_peak": round(14 * d * sum(pairs[b] for b in branch_ms) / (total * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                    "kernel_ms": {k_: round(v_, 3) for k_, v_ in ks.items()}}
            print(json.dumps(line), flush=True)


# workloads that run the forward pass only (the configuration says so)
FORWARD_ONLY = ("g64",)


def load_workload(name, heads=None):
    from paper_2505_17412_amd import inputs
    if name == "batch4":
        return inputs.make_batch_workload()
    over = {}
    if heads:
        h = [int(t) for t in heads.split(",")]
        over = dict(hq=h[0], hkv=h[1], d=h[2])
    return inputs.make_workload(name, **over)


def bench_workload(name, args, steps, warmup, cpu_seconds):
    """The benchmark line of one workload: whole-step time, per-kernel HIP-event times, roofline position of the
    dominant kernel and the oracle timed on a bounded query sample."""
    import numpy as np
    import torch
    from paper_2505_17412_amd import harness as util, ssa

    wl = load_workload(name, args.heads)
    bwd = name not in FORWARD_ONLY
    n, hq, hkv, d, T = wl.n_tokens, wl.n_heads_q, wl.n_heads_kv, wl.head_dim, wl.topk
    torch.cuda.set_device(0)
    p, blk = util.build_blocks_gpu(wl)
    t0 = time.perf_counter()
    for _ in range(3):
        util.build_blocks_gpu(wl)[1].destroy()
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) / 3 * 1e3

    q, k, v, g, do = (util.to_dev(a, wl.dtype) for a in (wl.q, wl.k, wl.v, wl.gates, wl.dout))
    out = torch.empty_like(q)
    ob = torch.empty((3,) + tuple(q.shape), dtype=q.dtype, device="cuda")
    lse = torch.empty((3, n, hq), dtype=torch.float32, device="cuda")
    idx = torch.empty((n, hkv, T), dtype=torch.int32, device="cuda")
    dq, dk, dv, dg = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v), torch.empty_like(g)
    wsf = torch.empty(ssa.ssa_workspace_bytes(p, blk, False), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(ssa.ssa_workspace_bytes(p, blk, True) if bwd else 16, dtype=torch.uint8, device="cuda")

    def fwd():
        ssa.ssa_forward(p, blk, q, k, v, g, out, lse, idx, ob, wsf)

    def bwd_pass():
        ssa.ssa_backward(p, blk, q, k, v, g, ob, lse, idx, do, dq, dk, dv, dg, wsb)

    def step():
        fwd()
        if bwd:
            bwd_pass()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3

    # forward / backward split (separate loops, HIP events on the launch stream)
    def timed(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    reps = max(3, steps // 2)
    fwd_ms = timed(fwd, reps)
    bwd_ms = timed(bwd_pass, reps) if bwd else None

    # per-kernel durations over the same steps, HIP events recorded by the library on the launch stream
    ssa.ssa_profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    prof = ssa.ssa_profile_get()
    ssa.ssa_profile_enable(False)
    kern_ms = {nm: tot / cnt for nm, (tot, cnt) in prof.items()}
    if "generic_path" in prof:  # one record per call (forward, backward): report the step's total
        kern_ms["generic_path"] = prof["generic_path"][0] / steps

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)  # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    arrays = {nm: blk.export(nm).cpu().numpy() for nm in ("perm", "tok_win", "win_start", "cmp_batch", "slc_start")}
    pairs = algorithmic_flops(wl, arrays, idx.cpu().numpy())
    all_pairs = pairs["cmp"] + pairs["slc"] + pairs["win"]
    # algorithmic FLOPs per kernel: forward 2 contractions (4d per pair); backward 5 (10d): S, dP, dQ booked on the
    # dQ kernel (6d), dV, dK on the dK/dV kernels (4d); recomputed scores are not counted
    kflops = {
        "cmp_fwd_scores_topk": 4 * d * pairs["cmp"], "slc_fwd": 4 * d * pairs["slc"], "win_fwd": 4 * d * pairs["win"],
        "bwd_dq_cmp_win": 6 * d * (pairs["cmp"] + pairs["win"]), "bwd_dq_slc": 6 * d * pairs["slc"], "bwd_dkv_cmp": 4 * d * pairs["cmp"], "bwd_dkv_slc": 4 * d * pairs["slc"],
        "bwd_dkv_win": 4 * d * pairs["win"], "generic_path": (14 if bwd else 4) * d * all_pairs,
    }
    dom = max(kern_ms, key=kern_ms.get) if kern_ms else None
    roofline = None
    if dom is not None and dom in kflops:
        ach = kflops[dom] / (kern_ms[dom] * 1e-3) / 1e12
        # a committed traffic figure covers the named workload in its own head shape only
        traffic, source = recorded_traffic(dom, name, d) if not args.heads else (None, None)
        # the generic kernels (fp32 problems, shapes the MFMA kernels do not cover) do their contractions on the
        # vector ALU: priced against the fp32 vector peak
        generic = dom == "generic_path"
        peak = FP32_VECTOR_PEAK_TFLOPS if generic else MFMA_BF16_PEAK_TFLOPS
        roofline = {"bound": "alu" if generic else "mfma", "kernel": dom, "achieved": round(ach, 2), "peak": peak,
                    "unit": "TFLOP/s", "frac": round(ach / peak, 4),
                    "traffic": traffic, "traffic_source": source, "kernel_ms": round(kern_ms[dom], 4)}
    total_flops = (14 if bwd else 4) * d * all_pairs
    # HBM-bound helper: gather + mean pool of K and V, priced at its algorithmic bytes (K, V read once, pooled rows
    # written once); the sorted copies the kernel also writes are this design's own extra traffic
    n_cmp = blk.counts()[0]
    prep_bytes = 2 * (n + n_cmp) * hkv * d * 2
    prep_gbps = round(prep_bytes / (kern_ms["prep_sort_pool"] * 1e-3) / 1e9, 1) if kern_ms.get("prep_sort_pool") else None

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ssa_oracle
        from oracle.ssa_oracle import oracle_for
        orc = oracle_for(wl)

        def oracle_step(sub):
            f = orc.forward(wl.q, wl.k, wl.v, wl.gates, queries=sub)
            if bwd:
                orc.backward(wl.q, wl.k, wl.v, wl.gates, wl.dout, f.topk_idx, out_branch=f.out_branch, queries=sub)

        probe = np.arange(0, n, max(1, n // 256), dtype=np.int32)[:256]
        oracle_step(probe[:32])  # first call pays library load and thread start-up
        t0 = time.perf_counter()
        oracle_step(probe)
        per_q = (time.perf_counter() - t0) / len(probe)
        ns = int(min(n, max(64, cpu_seconds / max(per_q, 1e-9))))
        sub = np.arange(0, n, max(1, n // ns), dtype=np.int32)[:ns]
        t0 = time.perf_counter()
        oracle_step(sub)
        dt = time.perf_counter() - t0
        what = "fwd+bwd" if bwd else "fwd"
        cpu = {"value": round(len(sub) / dt, 2), "unit": "tokens/s", "cores": ssa_oracle.n_threads(), "kind": "oracle",
               "sample": f"{what} of {len(sub)} evenly spaced query tokens of the same {n}-token workload, {dt:.1f} s wall",
               "seconds": round(dt, 2)}

    passes = "fwd+bwd" if bwd else "fwd"
    shape = (f"{wl.n_batch} union-of-primitives shells" if wl.n_batch > 1 else "union-of-primitives shell")
    line = {
        "metric": f"SSA {passes} tokens/sec", "value": round(n / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {shape} on a {wl.grid}^3 grid, N={n} tokens, Hq={hq}, "
                               f"Hkv={hkv}, d={d}, m_cmp/m_slc/m_win={wl.m_cmp}/{wl.m_slc}/{wl.m_win}, top-k={T}, {passes}",
                   "n_tokens": n, "n_batch": wl.n_batch, "blocks_cmp_slc_win": list(blk.counts())},
        "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4) if bwd else None, "build_blocks_ms": round(build_ms, 3),
        "tokens_per_s_incl_build_blocks": round(n / ((ms + build_ms) * 1e-3), 1),
        "prep_sort_pool_algorithmic_gbps": prep_gbps,
        "algorithmic_tflop_per_step": round(total_flops / 1e12, 4),
        "pairs_cmp_slc_win": [pairs["cmp"], pairs["slc"], pairs["win"]],
        "mfma_frac_whole_step": round(total_flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "kernel_ms": {k_: round(v_, 4) for k_, v_ in kern_ms.items()},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    blk.destroy()
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="g128", help="tiny | g64 (forward only) | g128 | batch4 | g128_thick")
    ap.add_argument("--all-configs", action="store_true", help="one benchmark line for each of the five workload configurations")
    ap.add_argument("--heads", default=None, help="HQ,HKV,D: another head shape on the same tokens (context figures; the default is the benchmark configuration)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="target CPU time of the oracle baseline leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known traffic, to scale rocprofv3 byte counters)")
    ap.add_argument("--gate", action="store_true", help="instead of the benchmark line: the gate predictor against the HBM roofline")
    ap.add_argument("--cmp-module", action="store_true",
                    help="instead of the benchmark line: the learned compression module alone and inside a training step")
    ap.add_argument("--ablation", action="store_true", help="instead of the benchmark line: the stress workload, top-k x window sweep with per-branch figures")
    ap.add_argument("--layer", action="store_true", help="instead of the benchmark line: a full SSA attention layer, forward + backward")
    ap.add_argument("--learned-cmp", action="store_true", help="with --layer: the learned compression module instead of the mean pool")
    ap.add_argument("--linear", action="store_true", help="instead of the benchmark line: the layer's linear projections against the MFMA roofline")
    ap.add_argument("--seq1d", action="store_true", help="instead of the benchmark line: the kernels on a one-dimensional (sequence) partition")
    ap.add_argument("--dense-sweep", action="store_true",
                    help="instead of the benchmark line: sparse path against dense attention over 2.6k-124k tokens")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.dense_sweep:
        dense_sweep(args)
        return
    if args.seq1d:
        seq1d_bench(args)
        return
    if args.linear:
        linear_bench(args)
        return
    if args.layer:
        layer_bench(args)
        return
    if args.ablation:
        ablation_sweep(args)
        return
    if args.cmp_module:
        cmp_module_bench(args)
        return
    if args.gate:
        gate_bench(args)
        return

    if args.all_configs:
        # the five workload configurations, one JSON line each (forward only where the configuration says so); fewer
        # timed steps and a smaller oracle sample than the default line so the whole table stays within minutes
        for name in ("tiny", "g64", "g128", "batch4", "g128_thick"):
            steps = args.steps if name in ("tiny", "g64", "g128") else max(3, args.steps // 4)
            print(json.dumps(bench_workload(name, args, steps, max(2, args.warmup // 2), args.cpu_seconds / 4)), flush=True)
        return
    print(json.dumps(bench_workload(args.workload, args, args.steps, args.warmup, args.cpu_seconds)), flush=True)


if __name__ == "__main__":
    main()
