"""GPU: ssa_forward / ssa_backward / ssa_topk_from_scores against the fp64 oracle, element by element.

Tolerances (relative to max|reference| of each tensor): bf16 2e-2 max / 1e-3 mean, fp32 1e-5 both.
Selected sets: equal to the oracle's, except that blocks whose oracle score lies within a relative margin
(2e-3 bf16, 1e-5 fp32) of the T-th best may swap; outputs are compared against the oracle run on the HIP
path's own selected sets (the selection is an explicit input of Algorithm 1).
"""
import numpy as np
import pytest

from oracle.ssa_oracle import oracle_for
from paper_2505_17412_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu


def full_parity(wl, backward=True, queries=None, tol_scale=1.0):
    print("parity", wl.name, wl.n_tokens, wl.dtype, wl.n_heads_q, wl.n_heads_kv, wl.head_dim, flush=True)
    orc = oracle_for(wl)
    dout = wl.dout
    if queries is not None:
        dout = np.zeros_like(wl.dout)
        dout[queries] = wl.dout[queries]
    g = util.run_gpu(wl, backward=backward, dout=dout)
    sel = slice(None) if queries is None else queries
    ref_own = orc.forward(wl.q, wl.k, wl.v, wl.gates, queries=queries, want_scores=True)
    ndiff = util.check_topk(g.topk_idx, ref_own, orc, wl.dtype, queries=queries)
    ref = orc.forward(wl.q, wl.k, wl.v, wl.gates, queries=queries, topk_idx=g.topk_idx)
    errs = {}
    errs["out"] = util.assert_close(g.out[sel], ref.out[sel], wl.dtype, "out", tol_scale)
    for b, nm in enumerate(("cmp", "slc", "win")):
        errs["out_" + nm] = util.assert_close(g.out_branch[b][sel], ref.out_branch[b][sel], wl.dtype, "out_" + nm, tol_scale)
        errs["lse_" + nm] = util.assert_close(g.lse[b][sel], ref.lse[b][sel], wl.dtype, "lse_" + nm, tol_scale)
    if backward:
        rb = orc.backward(wl.q, wl.k, wl.v, wl.gates, dout, g.topk_idx, out_branch=ref.out_branch, queries=queries)
        errs["dq"] = util.assert_close(g.dq[sel], rb.dq[sel], wl.dtype, "dq", tol_scale)
        errs["dk"] = util.assert_close(g.dk, rb.dk, wl.dtype, "dk", tol_scale)
        errs["dv"] = util.assert_close(g.dv, rb.dv, wl.dtype, "dv", tol_scale)
        errs["dgates"] = util.assert_close(g.dgates[sel], rb.dgates[sel], wl.dtype, "dgates", tol_scale)
    print("  topk rows differing:", ndiff, " errors:", {k: f"{v[0]:.1e}/{v[1]:.1e}" for k, v in errs.items()}, flush=True)
    return ndiff, errs


def test_tiny_fp32_full():
    """Config "tiny": 32^3 grid, three spheres, fp32, 4 heads (2 KV heads), d=32, T=4."""
    ndiff, _ = full_parity(inputs.make_workload("tiny"))
    assert ndiff == 0


@pytest.mark.parametrize("hq,hkv", [(4, 4), (4, 1), (8, 2)])
def test_tiny_fp32_head_groupings(hq, hkv):
    wl = inputs.make_workload("tiny", hq=hq, hkv=hkv, seed=1011)
    full_parity(wl, queries=np.arange(0, wl.n_tokens, 3, dtype=np.int32))


@pytest.mark.parametrize("seed,grid,n,hq,hkv,d,m,topk,dtype", [
    (11, 16, (300, 1, 170), 4, 2, 16, (2, 4, 4), 3, "f32"),
    (12, 16, (257,), 8, 1, 64, (2, 4, 8), 40, "f32"),      # T larger than the block count: -1 padding
    (13, 32, (700, 650), 16, 2, 64, (4, 8, 8), 4, "bf16"),
    (14, 32, (900,), 16, 1, 64, (4, 8, 4), 6, "bf16"),
    (15, 32, (640,), 16, 2, 128, (4, 8, 8), 5, "bf16"),
    (16, 16, (500,), 4, 4, 32, (2, 4, 4), 3, "bf16"),
    (18, 32, (800, 450), 24, 3, 64, (4, 8, 8), 5, "bf16"),  # three KV heads: rows the 16-byte pooling kernel does not take
    (17, 8, (400,), 4, 2, 24, (1, 2, 2), 2, "f32"),        # duplicates allowed below, odd head_dim
])
def test_random_points(seed, grid, n, hq, hkv, d, m, topk, dtype):
    wl = inputs.random_points_workload(seed, grid, n, hq, hkv, d, m, topk, dtype, allow_duplicates=(seed == 17))
    full_parity(wl)


def test_topk_from_scores_is_bit_exact():
    """The decision alone, on the oracle's fp32 scores plus planted ties, must match exactly."""
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.make_workload("tiny", topk=6)
    orc = oracle_for(wl)
    f = orc.forward(wl.q, wl.k, wl.v, wl.gates, want_scores=True)
    sc = f.scores.copy()
    sc[::3] = np.round(sc[::3] * 8) / 8            # many exact ties
    sc[1::7, :, :5] = 0.0
    rng = np.random.default_rng(0)
    sc[2::11] = rng.standard_normal(sc[2::11].shape).astype(np.float32)  # negative scores are ordered too
    expect = orc.topk_from_scores(sc)
    p, blk = util.build_blocks_gpu(wl)
    got = torch.full((wl.n_tokens, wl.n_heads_kv, wl.topk), -9, dtype=torch.int32, device="cuda")
    ssa.ssa_topk_from_scores(p, blk, torch.from_numpy(sc).cuda(), got)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), expect)
    # untouched scores reproduce the forward pass's own sets
    ssa.ssa_topk_from_scores(p, blk, torch.from_numpy(f.scores).cuda(), got)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), f.topk_idx)


def test_zero_queries_select_by_child_count():
    """Q = 0 makes the compression softmax uniform: the selected set is the closed form of eq. (6)."""
    wl = inputs.make_workload("tiny", topk=6)
    wl.q[:] = 0
    orc = oracle_for(wl)
    g = util.run_gpu(wl, backward=False)
    children = np.diff(orc.blocks.slc_child_start)
    expect = np.array(sorted(sorted(range(len(children)), key=lambda j: (-int(children[j]), j))[:6]), dtype=np.int32)
    assert np.all(g.topk_idx == expect[None, None, :])


def test_validation_on_gpu():
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.random_points_workload(1, 8, (40,), 4, 2, 16, (2, 4, 4), 2)
    p, blk = util.build_blocks_gpu(wl)
    q, k, v, g = (util.to_dev(a, "f32") for a in (wl.q, wl.k, wl.v, wl.gates))
    out = torch.zeros_like(q)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_forward(p, blk, q, k, v, g, out, workspace=small)
    assert e.value.status == -7
    p2 = util.params_of(wl)
    p2.n_tokens = 39
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_forward(p2, blk, q, k, v, g, out)
    assert e.value.status == -10
    # a tensor that does not start on a 16-byte boundary is refused before anything is launched
    shifted = torch.zeros(q.numel() + 1, dtype=q.dtype, device="cuda")[1:].view(q.shape)
    assert shifted.data_ptr() % 16 == 4
    for args in ((shifted, k, v, g, out), (q, k, v, g, shifted)):
        with pytest.raises(ssa.SSAError) as e:
            ssa.ssa_forward(p, blk, *args)
        assert e.value.status == -11
    p3 = util.params_of(wl)
    p3.n_heads_kv = 3
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_forward(p3, blk, q, k, v, g, out)
    assert e.value.status == -4
    p4 = util.params_of(wl)
    p4.head_dim = 20
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_forward(p4, blk, q, k, v, g, out)
    assert e.value.status == -8
    assert torch.all(out == 0)  # nothing was written
    ssa.ssa_forward(p, blk, q, k, v, g, out)  # inference call: optional outputs omitted
    torch.cuda.synchronize()
    ref = oracle_for(wl).forward(wl.q, wl.k, wl.v, wl.gates)
    util.assert_close(util.to_np(out), ref.out, "f32", "out")


def test_g64_bf16_forward_sampled():
    """Config "g64": 64^3 grid, ~11k tokens, bf16, 16 heads (2 KV heads), d=64, T=8, forward; every 8th query."""
    wl = inputs.make_workload("g64")
    full_parity(wl, backward=False, queries=np.arange(0, wl.n_tokens, 8, dtype=np.int32))


def test_g128_bf16_forward_backward_sampled():
    """Config "g128" (the benchmark workload): 128^3 grid, ~62k tokens, bf16, 16 heads (2 KV heads), d=64, T=16.
    The oracle visits every 97th query; dO is zero elsewhere (backward is linear in dO), so dK/dV compare in full."""
    wl = inputs.make_workload("g128")
    full_parity(wl, backward=True, queries=np.arange(5, wl.n_tokens, 97, dtype=np.int32))


def test_batch_of_four_shapes_sampled():
    """Variable-length batch: four 128^3 shapes (20k-70k tokens each) with batch offsets, bf16, 16 heads, d=64, T=16.
    Every key set must stay inside the query's own item."""
    wl = inputs.make_batch_workload()
    full_parity(wl, backward=True, queries=np.arange(11, wl.n_tokens, 389, dtype=np.int32))


@pytest.mark.parametrize("topk,m_win", [(8, 4), (8, 8), (16, 4), (16, 8), (32, 4), (32, 8)])
def test_g128_thick_d128_sampled(topk, m_win):
    """Stress config: thick shell (~150k tokens), head_dim 128, every point of the top-k x window sweep."""
    wl = inputs.make_workload("g128_thick", topk=topk, m=(4, 8, m_win))
    full_parity(wl, backward=True, queries=np.arange(3 + topk + m_win, wl.n_tokens, 613, dtype=np.int32))


@pytest.mark.parametrize("which", ["g64_bf16_matrix_cores", "tiny_f32_generic", "bf16_two_heads_per_kv_head"])
def test_forward_backward_are_deterministic(which):
    """Two runs on the same inputs give bit-identical outputs: no floating-point sum depends on scheduling, on the
    matrix-core path (h_s = 8), on the fp32 path and on the bf16 shapes whose backward runs on the fp32-arithmetic
    kernels (h_s = 2)."""
    if which == "g64_bf16_matrix_cores":
        wl = inputs.make_workload("g64")
    elif which == "tiny_f32_generic":
        wl = inputs.make_workload("tiny")
    else:
        wl = inputs.random_points_workload(44, 32, (1500, 900), 8, 4, 64, (4, 8, 8), 5, "bf16")
    a = util.run_gpu(wl, backward=True)
    b = util.run_gpu(wl, backward=True)
    for name in ("out", "lse", "topk_idx", "dq", "dk", "dv", "dgates"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name


def test_bf16_inference_call_without_optional_outputs():
    """ssa_forward with lse / topk_idx / out_branch = NULL (inference) writes the same `out` as the training call."""
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.random_points_workload(21, 32, (900, 500), 16, 2, 64, (4, 8, 8), 6, "bf16")
    full = util.run_gpu(wl, backward=False)
    p, blk = util.build_blocks_gpu(wl)
    q, k, v, g = (util.to_dev(a, "bf16") for a in (wl.q, wl.k, wl.v, wl.gates))
    out = torch.zeros_like(q)
    ssa.ssa_forward(p, blk, q, k, v, g, out)
    torch.cuda.synchronize()
    assert np.array_equal(util.to_np(out), full.out)


def test_whole_grid_window_is_dense_attention_on_gpu():
    """A window covering the whole grid makes the window branch plain dense attention (window paragraph): the same
    kernels then serve as a dense variable-length flash attention, forward and backward."""
    wl = inputs.random_points_workload(22, 16, (1500, 700), 16, 2, 64, (4, 8, 16), 4, "bf16")
    orc = oracle_for(wl)
    assert orc.blocks.n_blocks["win"] == 2  # one window per batch item
    gates = np.zeros_like(wl.gates)
    gates[..., 2] = 1.0
    wl.gates = gates
    g = util.run_gpu(wl, backward=True)
    qf, kf, vf = (a.astype(np.float64) for a in (wl.q, wl.k, wl.v))
    for b in range(2):
        sl = slice(int(wl.batch_offsets[b]), int(wl.batch_offsets[b + 1]))
        for h in (0, 9, 15):
            s = (qf[sl, h] @ kf[sl, h // 8].T) * orc.scale
            p = np.exp(s - s.max(1, keepdims=True))
            p /= p.sum(1, keepdims=True)
            util.assert_close(g.out[sl, h], p @ vf[sl, h // 8], "bf16", f"dense out item {b} head {h}")
    ref = orc.forward(wl.q, wl.k, wl.v, wl.gates, topk_idx=g.topk_idx)
    rb = orc.backward(wl.q, wl.k, wl.v, wl.gates, wl.dout, g.topk_idx, out_branch=ref.out_branch)
    for name, got, want in (("dq", g.dq, rb.dq), ("dk", g.dk, rb.dk), ("dv", g.dv, rb.dv)):
        util.assert_close(got, want, "bf16", name)


def test_shifted_windows_are_the_window_kernels_on_shifted_coordinates():
    """Shifted 3D windows (the VAE's window attention alternates plain and half-window-shifted partitions, section 3.1)
    need no kernel of their own: a second block handle built on coordinates moved by half a window partitions the
    tokens into the shifted windows.  The window branch is checked against dense attention inside windows whose ids
    are computed here from floor((c + m/2) / m), not by the oracle's block builder."""
    import dataclasses
    base = inputs.random_points_workload(23, 16, (1300, 900), 16, 2, 64, (4, 8, 8), 4, "bf16")
    shift = base.m_win // 2
    wl = dataclasses.replace(base, coords=base.coords + shift, grid=base.grid + base.m_win)
    gates = np.zeros_like(wl.gates)
    gates[..., 2] = 1.0
    wl.gates = gates
    g = util.run_gpu(wl, backward=False)
    item = np.searchsorted(wl.batch_offsets, np.arange(wl.n_tokens), side="right") - 1
    w = (base.coords + shift) // base.m_win
    wid = ((item * 4 + w[:, 0]) * 4 + w[:, 1]) * 4 + w[:, 2]
    plain = base.coords // base.m_win
    assert len(np.unique(wid)) != len(np.unique(((item * 4 + plain[:, 0]) * 4 + plain[:, 1]) * 4 + plain[:, 2]))
    qf, kf, vf = (a.astype(np.float64) for a in (wl.q, wl.k, wl.v))
    scale = 1.0 / np.sqrt(wl.head_dim)
    for win in np.unique(wid)[::7]:
        rows = np.nonzero(wid == win)[0]
        for h in (0, 11):
            s = (qf[rows, h] @ kf[rows, h // 8].T) * scale
            p = np.exp(s - s.max(1, keepdims=True))
            p /= p.sum(1, keepdims=True)
            util.assert_close(g.out[rows, h], p @ vf[rows, h // 8], "bf16", f"shifted window {win} head {h}")


@pytest.mark.parametrize("seed,n,expect_blocks", [
    (31, (900,), (513, 1024)),     # selection blocks per item in (512, 1024]
    (32, (3000,), (1025, 4096)),   # more than 1024 selection blocks per item
])
def test_many_selection_blocks(seed, n, expect_blocks):
    """Sparse random points on a 64^3 grid with 4^3 selection blocks: the top-k search runs over hundreds to
    thousands of candidate blocks per item (every size class of the search routine is visited)."""
    wl = inputs.random_points_workload(seed, 64, n, 16, 2, 64, (2, 4, 4), 8, "bf16")
    ns = oracle_for(wl).blocks.n_blocks["slc"]
    assert expect_blocks[0] <= ns <= expect_blocks[1], ns
    full_parity(wl)


def test_many_blocks_over_many_items_sampled():
    """Twelve items with ~500 selection blocks each: more (KV head, block) keys than the chunk-ordering kernel copies
    into LDS, so its bisections run on global memory; every item small, queries sampled."""
    wl = inputs.random_points_workload(33, 32, (1500,) * 12, 16, 2, 64, (2, 4, 4), 6, "bf16")
    assert 2 * oracle_for(wl).blocks.n_blocks["slc"] > 8192
    full_parity(wl, queries=np.arange(3, wl.n_tokens, 9, dtype=np.int32))


@pytest.mark.parametrize("hq,hkv,d", [(8, 4, 64), (8, 2, 32), (2, 2, 128)])
def test_bf16_small_head_groups(hq, hkv, d):
    """bf16 with h_s = 2, 4 and 1 queries per KV head (8 or more token slots share one 16-column matrix tile)."""
    wl = inputs.random_points_workload(40 + hq + hkv, 32, (800, 333), hq, hkv, d, (4, 8, 8), 5, "bf16")
    full_parity(wl)


def test_empty_call_and_empty_batch_item():
    """N = 0 returns success without touching the outputs; a batch whose middle item is empty matches the oracle."""
    import torch
    from paper_2505_17412_amd import ssa
    wl0 = inputs.random_points_workload(1, 8, (0, 0), 4, 2, 16, (2, 4, 4), 2)
    p, blk = util.build_blocks_gpu(wl0)
    e = torch.empty((0, 4, 16), dtype=torch.float32, device="cuda")
    ekv = torch.empty((0, 2, 16), dtype=torch.float32, device="cuda")
    eg = torch.empty((0, 4, 3), dtype=torch.float32, device="cuda")
    ssa.ssa_forward(p, blk, e, ekv, ekv, eg, e)
    torch.cuda.synchronize()
    blk.destroy()
    wl = inputs.random_points_workload(33, 16, (300, 0, 211), 4, 2, 32, (2, 4, 4), 3, "f32")
    full_parity(wl)


def test_forward_backward_replay_from_a_hip_graph():
    """The training step records into a HIP graph (no allocation, no synchronisation, no memset nodes inside the
    library calls) and every replay, with eager work and synchronisations in between, reproduces the eager result
    bit for bit."""
    import torch
    from paper_2505_17412_amd import ssa
    # 4 800 tokens: large enough for the selection kernels to run in their own token order (built by kernels alone)
    wl = inputs.random_points_workload(23, 32, (3000, 1800), 16, 2, 64, (4, 8, 8), 6, "bf16")
    n, hq, hkv, d, T = wl.n_tokens, wl.n_heads_q, wl.n_heads_kv, wl.head_dim, wl.topk
    p, blk = util.build_blocks_gpu(wl)
    q, k, v, g, do = (util.to_dev(a, "bf16") for a in (wl.q, wl.k, wl.v, wl.gates, wl.dout))
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
    eager = [t.clone() for t in (out, lse, idx, dq, dk, dv, dg)]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                      # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for r in range(3):
        for t in (out, lse, dq, dk, dv, dg):
            t.fill_(float("nan"))   # eager work between the replays: the graph must rewrite every output
        idx.fill_(-5)
        wsf.random_(0, 255)
        wsb.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("out", "lse", "idx", "dq", "dk", "dv", "dgates"), (out, lse, idx, dq, dk, dv, dg), eager):
            assert torch.equal(got, want), (r, name)


@pytest.mark.parametrize("which", ["bf16_matrix_cores", "f32_generic"])
def test_backward_takes_selected_ids_in_any_order(which):
    """ssa_backward's contract for a caller-supplied I: distinct ids, the -1 padding at the end, any order.  The
    gradients with every row's ids shuffled must match those with the forward's ascending rows (the sums are taken in
    another order, so to the tolerance of the dtype, not bit for bit)."""
    if which == "bf16_matrix_cores":
        wl = inputs.random_points_workload(51, 32, (1400, 600), 16, 2, 64, (4, 8, 8), 6, "bf16")
    else:
        wl = inputs.random_points_workload(52, 16, (500, 300), 4, 2, 16, (2, 4, 4), 5, "f32")

    def shuffled(idx):
        rng = np.random.default_rng(7)
        out = idx.copy()
        for t in range(idx.shape[0]):
            for g in range(idx.shape[1]):
                nv = int(np.sum(idx[t, g] >= 0))
                out[t, g, :nv] = rng.permutation(idx[t, g, :nv])
        return out

    a = util.run_gpu(wl, backward=True)
    b = util.run_gpu(wl, backward=True, idx_for_backward=shuffled)
    assert np.array_equal(a.topk_idx, b.topk_idx)
    for name in ("dq", "dk", "dv", "dgates"):
        util.assert_close(getattr(b, name), getattr(a, name), wl.dtype, name)


@pytest.mark.parametrize("which", ["bf16_matrix_cores", "f32_generic"])
def test_gates_of_any_sign_and_zero(which):
    """Eq. (4) is linear in the gates, and the interface takes any real gate tensor (the gate predictor's sigmoid is
    only one producer): negative gates, and gates that are exactly zero for a whole branch of some tokens, must give the
    oracle's output and gradients (a zero gate: no contribution to out, dq, dk, dv, but a dgates entry all the same)."""
    if which == "bf16_matrix_cores":
        wl = inputs.random_points_workload(61, 32, (1100, 500), 16, 2, 64, (4, 8, 8), 5, "bf16")
    else:
        wl = inputs.random_points_workload(62, 16, (400, 250), 4, 2, 16, (2, 4, 4), 4, "f32")
    rng = np.random.default_rng(5)
    gates = rng.standard_normal(wl.gates.shape).astype(np.float32)
    gates[rng.random(wl.gates.shape) < 0.15] = 0.0
    gates[::7, :, 1] = 0.0  # every 7th token: selection branch switched off for all heads
    wl.gates = inputs.round_to_bf16(gates) if wl.dtype == "bf16" else gates
    assert (wl.gates < 0).any() and (wl.gates == 0).any()
    full_parity(wl)


@pytest.mark.parametrize("seed,grid,n,hq,hkv,d,m,topk", [
    (167765, 64, (73,), 16, 1, 64, (1, 2, 4), 1),
    (7, 32, (150, 90), 8, 1, 64, (1, 2, 4), 1),
])
def test_softmaxes_over_one_or_two_keys(seed, grid, n, hq, hkv, d, m, topk):
    """A few dozen scattered tokens, one-voxel compression blocks, one selected block: most selection and window
    softmaxes run over one or two keys, where dP equals delta up to rounding and dS = P (dP - delta) is what the
    roundings leave.  The two sums must then be taken over the same rounded numbers (the backward kernels that read the
    gate-weighted dO rows subtract a delta formed from those same rows), or dK drifts out of the tolerance."""
    full_parity(inputs.random_points_workload(seed, grid, n, hq, hkv, d, m, topk, "bf16"))
