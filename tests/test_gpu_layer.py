"""GPU: the full SSA attention layer (projections, gate predictor, attention, output projection) against the chained
fp64 oracle.  Forward is checked stage by stage: every stage of the oracle is fed the bf16 tensor the HIP path saved for
the stage before, so each comparison sees one stage's arithmetic (tolerances of the attention path).  Backward is
checked end to end against the oracle chain started from the saved activations (the intermediate gradients dO, dq, dk,
dv, dgates are bf16 on the HIP side; the same tolerances still hold for every result)."""
import numpy as np
import pytest

from oracle.gate import gate_forward
from oracle.layer import LayerForward, LayerWeights, layer_backward
from oracle.linear import linear_forward
from oracle.ssa_oracle import oracle_for
from paper_2505_17412_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu

W_NAMES = ("wq", "wk", "wv", "wg", "bg", "wo", "bq", "bk", "bv", "bo")


def make_weights(rng, dm, cq, ckv, hq, biases):
    r = inputs.round_to_bf16
    g = lambda *s: rng.standard_normal(s).astype(np.float32)
    w = dict(wq=r(g(cq, dm) / np.sqrt(dm)), wk=r(g(ckv, dm) / np.sqrt(dm)), wv=r(g(ckv, dm) / np.sqrt(dm)),
             wg=r(g(dm, 3 * hq) / np.sqrt(dm)), bg=r(g(3 * hq)), wo=r(g(dm, cq) / np.sqrt(cq)))
    if biases:
        w.update(bq=r(g(cq) * 0.1), bk=r(g(ckv) * 0.1), bv=r(g(ckv) * 0.1), bo=r(g(dm) * 0.1))
    return w


@pytest.mark.parametrize("seed,grid,n,hq,hkv,d,dm,topk,biases", [
    (81, 16, (700, 450), 16, 2, 64, 256, 4, True),
    (82, 32, (1500,), 16, 2, 64, 1024, 6, False),     # the paper's layer shape: hidden 1024, 16 heads of 64, 2 KV heads
    (83, 16, (300, 0, 333), 8, 1, 128, 128, 3, True),
])
def test_layer_forward_backward(seed, grid, n, hq, hkv, d, dm, topk, biases):
    import torch
    from paper_2505_17412_amd import ssa
    print("layer", seed, n, hq, hkv, d, dm, flush=True)
    wl = inputs.random_points_workload(seed, grid, n, hq, hkv, d, (4, 8, 8), topk, "bf16")
    N, cq, ckv = wl.n_tokens, hq * d, hkv * d
    rng = np.random.default_rng(seed)
    r = inputs.round_to_bf16
    x = r(rng.standard_normal((N, dm)).astype(np.float32))
    dy = r(rng.standard_normal((N, dm)).astype(np.float32))
    w = make_weights(rng, dm, cq, ckv, hq, biases)
    p, blk = util.build_blocks_gpu(wl)
    tw = {k: util.to_dev(v, "bf16") for k, v in w.items()}
    tx, tdy = util.to_dev(x, "bf16"), util.to_dev(dy, "bf16")
    nbytes, offs = ssa.ssa_layer_saved_bytes(p)
    saved = torch.zeros(nbytes + 256, dtype=torch.uint8, device="cuda")
    y = torch.full((N, dm), float("nan"), dtype=torch.bfloat16, device="cuda")
    ssa.ssa_layer_forward(p, blk, tx, tw, y, saved)
    torch.cuda.synchronize()
    base = (-saved.data_ptr()) % 256

    def view(name, shape, dtype):
        nb = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        return saved[base + offs[name]: base + offs[name] + nb].view(dtype).view(*shape)

    q = util.to_np(view("q", (N, hq, d), torch.bfloat16))
    k = util.to_np(view("k", (N, hkv, d), torch.bfloat16))
    v = util.to_np(view("v", (N, hkv, d), torch.bfloat16))
    gates = util.to_np(view("gates", (N, hq, 3), torch.bfloat16))
    o = util.to_np(view("o", (N, hq, d), torch.bfloat16))
    ob = util.to_np(view("out_branch", (3, N, hq, d), torch.bfloat16))
    lse = util.to_np(view("lse", (3, N, hq), torch.float32))
    idx = util.to_np(view("topk_idx", (N, hkv, topk), torch.int32))
    # ---- forward, stage by stage
    util.assert_close(q.reshape(N, cq), linear_forward(x, w["wq"], w.get("bq")), "bf16", "q")
    util.assert_close(k.reshape(N, ckv), linear_forward(x, w["wk"], w.get("bk")), "bf16", "k")
    util.assert_close(v.reshape(N, ckv), linear_forward(x, w["wv"], w.get("bv")), "bf16", "v")
    util.assert_close(gates.reshape(N, 3 * hq), gate_forward(x, w["wg"], w["bg"]), "bf16", "gates")
    orc = oracle_for(wl)
    own = orc.forward(q, k, v, gates, want_scores=True)
    util.check_topk(idx, own, orc, "bf16")
    ref = orc.forward(q, k, v, gates, topk_idx=idx)
    util.assert_close(o, ref.out, "bf16", "attention out")
    for b in range(3):
        util.assert_close(ob[b], ref.out_branch[b], "bf16", f"out_branch {b}")
        util.assert_close(lse[b], ref.lse[b], "bf16", f"lse {b}")
    util.assert_close(util.to_np(y), linear_forward(o.reshape(N, cq), w["wo"], w.get("bo")), "bf16", "y")
    # ---- backward, end to end from the saved activations
    g_names = ["dwq", "dwk", "dwv", "dwg", "dbg", "dwo"] + (["dbq", "dbk", "dbv", "dbo"] if biases else [])
    grads = {nm: torch.full(w[nm[1:]].shape, float("nan"), dtype=torch.float32, device="cuda") for nm in g_names}
    dx = torch.full((N, dm), float("nan"), dtype=torch.bfloat16, device="cuda")
    ssa.ssa_layer_backward(p, blk, tx, tw, saved, tdy, dx, grads)
    torch.cuda.synchronize()
    lw = LayerWeights(**{nm: w.get(nm) for nm in W_NAMES})
    ref.out = o  # the oracle chain starts from what the HIP path saved (and rounded)
    ref.out_branch = ob
    rb = layer_backward(orc, x, lw, LayerForward(q, k, v, gates, ref, None), dy)
    errs = {"dx": util.assert_close(util.to_np(dx), rb["dx"], "bf16", "dx")}
    for nm in g_names:
        if nm == "dbk":
            # Adding one vector to every key shifts all scores of a query alike and leaves every softmax unchanged: the
            # exact gradient is zero, and both sides hold only rounding noise of the column sums of dk.
            bound = 2e-3 * np.abs(rb["dk"]).reshape(N, ckv).sum(axis=0)
            assert np.all(np.abs(util.to_np(grads[nm])) <= bound), nm
            continue
        errs[nm] = util.assert_close(util.to_np(grads[nm]), rb[nm], "bf16", nm)
    print("  errors:", {k_: f"{v_[0]:.1e}/{v_[1]:.1e}" for k_, v_ in errs.items()}, flush=True)


def test_layer_with_learned_compression_module():
    """The layer with the learned compression module on keys and values (Sparse 3D Compression, eq. (5)) in place of
    the mean pool: forward against the oracle chain fed the saved q, k, v, gates; backward end to end, including the
    six parameter gradients of the two modules."""
    import torch
    from oracle.cmp_module import CompressionModule
    from oracle.layer import block_tokens
    from paper_2505_17412_amd import ssa
    seed, hq, hkv, d, dm, topk = 84, 16, 2, 64, 256, 5
    wl = inputs.random_points_workload(seed, 32, (1300, 800), hq, hkv, d, (4, 8, 8), topk, "bf16")
    N, cq, ckv = wl.n_tokens, hq * d, hkv * d
    rng = np.random.default_rng(seed)
    r = inputs.round_to_bf16
    gn = lambda *s: rng.standard_normal(s).astype(np.float32)
    x, dy = r(gn(N, dm)), r(gn(N, dm))
    w = make_weights(rng, dm, cq, ckv, hq, True)
    for t in ("k", "v"):
        w["pe_" + t] = r(0.5 * gn(64, ckv))
        w["wc_" + t] = r(gn(27, ckv, ckv) / np.sqrt(9.0 * ckv))
        w["bc_" + t] = r(0.1 * gn(ckv))
    p, blk = util.build_blocks_gpu(wl)
    tw = {k: util.to_dev(v, "bf16") for k, v in w.items()}
    tx, tdy = util.to_dev(x, "bf16"), util.to_dev(dy, "bf16")
    nbytes, offs = ssa.ssa_layer_saved_bytes(p)
    saved = torch.zeros(nbytes + 256, dtype=torch.uint8, device="cuda")
    y = torch.full((N, dm), float("nan"), dtype=torch.bfloat16, device="cuda")
    ssa.ssa_layer_forward(p, blk, tx, tw, y, saved)
    torch.cuda.synchronize()
    base = (-saved.data_ptr()) % 256

    def view(name, shape, dtype):
        nb = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        return util.to_np(saved[base + offs[name]: base + offs[name] + nb].view(dtype).view(*shape))

    q, k, v = view("q", (N, hq, d), torch.bfloat16), view("k", (N, hkv, d), torch.bfloat16), view("v", (N, hkv, d), torch.bfloat16)
    gates, o = view("gates", (N, hq, 3), torch.bfloat16), view("o", (N, hq, d), torch.bfloat16)
    ob, idx = view("out_branch", (3, N, hq, d), torch.bfloat16), view("topk_idx", (N, hkv, topk), torch.int32)
    orc = oracle_for(wl)
    module = CompressionModule(wl.coords, wl.batch_offsets, wl.m_cmp, orc.blocks.ids["cmp"], orc.blocks.n_blocks["cmp"])
    lw = LayerWeights(**w)
    kc, vc = block_tokens(orc, module, k, v, lw)
    kc, vc = r(kc.astype(np.float32)), r(vc.astype(np.float32))  # the block tokens cross the boundary in bf16
    own = orc.forward(q, k, v, gates, want_scores=True, k_cmp=kc, v_cmp=vc)
    util.check_topk(idx, own, orc, "bf16")
    ref = orc.forward(q, k, v, gates, topk_idx=idx, k_cmp=kc, v_cmp=vc)
    util.assert_close(o, ref.out, "bf16", "attention out")
    pooled = orc.forward(q, k, v, gates, topk_idx=idx)
    assert np.abs(pooled.out_branch[0] - ref.out_branch[0]).max() > 0.05  # not the mean pool
    util.assert_close(util.to_np(y), linear_forward(o.reshape(N, cq), w["wo"], w["bo"]), "bf16", "y")
    # ---- backward
    g_names = ["d" + nm for nm in w]
    grads = {nm: torch.full(w[nm[1:]].shape, float("nan"), dtype=torch.float32, device="cuda") for nm in g_names}
    dx = torch.full((N, dm), float("nan"), dtype=torch.bfloat16, device="cuda")
    ssa.ssa_layer_backward(p, blk, tx, tw, saved, tdy, dx, grads)
    torch.cuda.synchronize()
    ref.out, ref.out_branch = o, ob
    rb = layer_backward(orc, x, lw, LayerForward(q, k, v, gates, ref, None, kc, vc), dy, module=module)
    errs = {"dx": util.assert_close(util.to_np(dx), rb["dx"], "bf16", "dx")}
    for nm in g_names:
        if nm == "dbc_k":
            # one vector added to every block-level key shifts all compression scores of a query alike: the exact
            # gradient is zero (the oracle's is not quite, it starts from the rounded out_branch the HIP path saved);
            # what is left on both sides is rounding of the column sums of dk_cmp
            bound = 2e-3 * np.abs(rb["dk_cmp"]).reshape(-1, ckv).sum(axis=0)
            assert np.all(np.abs(util.to_np(grads[nm]) - rb[nm]) <= bound), nm
            continue
        if nm == "dbk":
            # the selection and window parts of the column sums of dk cancel exactly (a vector added to every key
            # leaves those softmaxes unchanged); only the module's part survives, far below the terms' absolute sum,
            # which is what the rounding of dk scales with
            bound = 2e-3 * np.abs(rb["dk"]).reshape(N, ckv).sum(axis=0)
            assert np.all(np.abs(util.to_np(grads[nm]) - rb[nm]) <= bound), nm
            continue
        errs[nm] = util.assert_close(util.to_np(grads[nm]), rb[nm], "bf16", nm)
    print("  errors:", {k_: f"{v_[0]:.1e}/{v_[1]:.1e}" for k_, v_ in errs.items()}, flush=True)
    # some but not all of the module's pointers: refused
    bad = dict(tw)
    del bad["bc_v"]
    with pytest.raises(ssa.SSAError):
        ssa.ssa_layer_forward(p, blk, tx, bad, y, saved)


def test_layer_validation():
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.random_points_workload(5, 8, (64,), 4, 2, 32, (2, 4, 4), 2, "bf16")   # Hkv*d = 64: not a multiple of 128
    p, blk = util.build_blocks_gpu(wl)
    assert ssa.ssa_layer_workspace_bytes(p, blk, 128, False) == 0
    wl = inputs.random_points_workload(5, 8, (64,), 4, 2, 64, (2, 4, 4), 2, "bf16")
    p, blk = util.build_blocks_gpu(wl)
    assert ssa.ssa_layer_workspace_bytes(p, blk, 100, False) == 0                     # d_model not a multiple of 128
    assert ssa.ssa_layer_workspace_bytes(p, blk, 128, True) > 0
    x = torch.zeros((64, 128), dtype=torch.bfloat16, device="cuda")
    w = {k: x for k in ("wq", "wk", "wv", "wg", "bg", "wo")}
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_layer_forward(p, blk, x, w, x, torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -7


def test_layer_without_tokens():
    """No tokens: forward writes nothing, backward leaves zero parameter gradients."""
    import torch
    from paper_2505_17412_amd import ssa
    p = ssa.make_params(0, 2, 8, 2, 4, 4, 2, 4, 2, 64, "bf16")
    blk = ssa.ssa_build_blocks(p, torch.zeros((1, 3), dtype=torch.int32, device="cuda"),
                               torch.zeros(3, dtype=torch.int32, device="cuda"))
    dm, cq, ckv, hq = 128, 256, 128, 4
    z = lambda *s_: torch.zeros(s_, dtype=torch.bfloat16, device="cuda")
    w = dict(wq=z(cq, dm), wk=z(ckv, dm), wv=z(ckv, dm), wg=z(dm, 3 * hq), bg=z(3 * hq), wo=z(dm, cq))
    x = z(0, dm)
    saved = torch.empty(max(ssa.ssa_layer_saved_bytes(p)[0], 1), dtype=torch.uint8, device="cuda")
    module = dict(pe_k=z(8, ckv), wc_k=z(27, ckv, ckv), bc_k=z(ckv), pe_v=z(8, ckv), wc_v=z(27, ckv, ckv), bc_v=z(ckv))
    for weights in (w, dict(w, **module)):   # mean pool, then the learned compression module
        ssa.ssa_layer_forward(p, blk, x, weights, x, saved)
        grads = {"d" + k_: torch.full(v_.shape, float("nan"), dtype=torch.float32, device="cuda") for k_, v_ in weights.items()}
        ssa.ssa_layer_backward(p, blk, x, weights, saved, x, x, grads)
        torch.cuda.synchronize()
        for nm, t in grads.items():
            assert float(t.abs().max()) == 0.0, nm


def test_layer_step_replays_from_a_hip_graph():
    """The whole layer step, learned compression module included, records into a HIP graph (the library calls allocate
    nothing, synchronise nothing and record no memset nodes) and every replay, with eager work and synchronisations
    in between, reproduces the eager results bit for bit."""
    import torch
    from paper_2505_17412_amd import ssa
    hq, hkv, d, dm, topk = 16, 2, 64, 256, 6
    wl = inputs.random_points_workload(91, 32, (2900, 1700), hq, hkv, d, (4, 8, 8), topk, "bf16")
    N, cq, ckv = wl.n_tokens, hq * d, hkv * d
    p, blk = util.build_blocks_gpu(wl)
    gen = torch.Generator(device="cuda").manual_seed(91)
    rnd = lambda *s_, scale=1.0: (torch.randn(s_, generator=gen, device="cuda") * scale).bfloat16()
    x, dy = rnd(N, dm), rnd(N, dm)
    w = dict(wq=rnd(cq, dm, scale=dm ** -0.5), wk=rnd(ckv, dm, scale=dm ** -0.5), wv=rnd(ckv, dm, scale=dm ** -0.5),
             wg=rnd(dm, 3 * hq, scale=dm ** -0.5), bg=rnd(3 * hq), wo=rnd(dm, cq, scale=cq ** -0.5), bq=rnd(cq, scale=0.1),
             bk=rnd(ckv, scale=0.1), bv=rnd(ckv, scale=0.1), bo=rnd(dm, scale=0.1))
    for t in ("k", "v"):
        w.update({"pe_" + t: rnd(64, ckv, scale=0.5), "wc_" + t: rnd(27, ckv, ckv, scale=(9.0 * ckv) ** -0.5),
                  "bc_" + t: rnd(ckv, scale=0.1)})
    grads = {"d" + k_: torch.empty(v_.shape, device="cuda") for k_, v_ in w.items()}
    y, dx = torch.empty_like(x), torch.empty_like(x)
    saved = torch.empty(ssa.ssa_layer_saved_bytes(p)[0], dtype=torch.uint8, device="cuda")
    wsf = torch.empty(ssa.ssa_layer_workspace_bytes(p, blk, dm, False), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(ssa.ssa_layer_workspace_bytes(p, blk, dm, True), dtype=torch.uint8, device="cuda")

    def step():
        ssa.ssa_layer_forward(p, blk, x, w, y, saved, wsf)
        ssa.ssa_layer_backward(p, blk, x, w, saved, dy, dx, grads, wsb)

    step()
    torch.cuda.synchronize()
    outputs = dict(y=y, dx=dx, **grads)
    eager = {nm: t.clone() for nm, t in outputs.items()}
    assert all(bool(torch.isfinite(t.float()).all()) for t in eager.values())
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
        for t in outputs.values():
            t.fill_(float("nan"))   # eager work between the replays: the graph must rewrite every output
        for buf in (saved, wsf, wsb):
            buf.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for nm, t in outputs.items():
            assert torch.equal(t, eager[nm]), (r, nm)
