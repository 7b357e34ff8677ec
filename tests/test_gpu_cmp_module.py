"""GPU: the learned compression module (eq. (5)) and the attention entry points that take its output, against the
fp64 oracles, element by element.

Tolerances as for the attention path (relative to max|reference| of each tensor): 2e-2 max, 1e-3 mean; the module
rounds x + PE and the pooled gradient to bf16 before its matrix-core contractions, like every bf16 GEMM input.
"""
import numpy as np
import pytest

from oracle.cmp_module import CompressionModule
from oracle.ssa_oracle import oracle_for
from paper_2505_17412_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu


def draw_weights(seed, m, c):
    """Seeded module weights, rounded to bf16 (both sides get the rounded values)."""
    rng = np.random.default_rng(seed)
    r = inputs.round_to_bf16
    pe = r(0.5 * rng.standard_normal((m ** 3, c)).astype(np.float32))
    w = r((rng.standard_normal((27, c, c)) / np.sqrt(9.0 * c)).astype(np.float32))
    bias = r(0.1 * rng.standard_normal(c).astype(np.float32))
    return pe, w, bias


def module_oracle(wl):
    orc = oracle_for(wl)
    b = orc.blocks
    return orc, CompressionModule(wl.coords, wl.batch_offsets, wl.m_cmp, b.ids["cmp"], b.n_blocks["cmp"])


def gpu_module(wl, p, blk, x, pe, w, bias, dx_cmp=None, dx_init=None):
    import torch
    from paper_2505_17412_amd import ssa
    nc = blk.counts()[0]
    c = wl.n_heads_kv * wl.head_dim
    tx, tpe, tw, tb = (util.to_dev(a, "bf16") for a in (x, pe, w, bias))
    xc = torch.full((nc, wl.n_heads_kv, wl.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    ssa.ssa_compress_forward(p, blk, tx, tpe, tw, tb, xc)
    torch.cuda.synchronize()
    res = {"x_cmp": util.to_np(xc)}
    if dx_cmp is not None:
        dxa = util.to_dev(dx_init, "bf16")
        dpe = torch.full((wl.m_cmp ** 3, c), float("nan"), dtype=torch.float32, device="cuda")
        dw = torch.full((27, c, c), float("nan"), dtype=torch.float32, device="cuda")
        db = torch.full((c,), float("nan"), dtype=torch.float32, device="cuda")
        ssa.ssa_compress_backward(p, blk, tx, tpe, tw, tb, torch.from_numpy(np.ascontiguousarray(dx_cmp, dtype=np.float32)).cuda(),
                                  dxa, dpe, dw, db)
        torch.cuda.synchronize()
        res.update(dx=util.to_np(dxa), dpe=util.to_np(dpe), dw=util.to_np(dw), dbias=util.to_np(db))
    return res


@pytest.mark.parametrize("seed,grid,n,hkv,d,m", [
    (51, 16, (700,), 1, 32, (2, 4, 4)),
    (52, 16, (900, 1, 300), 2, 32, (4, 8, 8)),       # C = 64, a one-token item
    (53, 32, (2500, 1800), 2, 64, (4, 8, 8)),        # C = 128: the benchmark's channel count
    (54, 16, (1200,), 2, 128, (2, 4, 8)),            # C = 256
    (55, 8, (512,), 2, 64, (2, 4, 4)),               # every voxel of the grid active: all 27 neighbours exist inside
])
def test_module_forward_backward(seed, grid, n, hkv, d, m):
    wl = inputs.random_points_workload(seed, grid, n, 2 * hkv, hkv, d, m, 2, "bf16")
    orc, mod = module_oracle(wl)
    c = hkv * d
    pe, w, bias = draw_weights(seed, m[0], c)
    x = wl.k.reshape(wl.n_tokens, c)
    rng = np.random.default_rng(seed + 7)
    dxc = rng.standard_normal((orc.blocks.n_blocks["cmp"], c)).astype(np.float32)
    dx0 = inputs.round_to_bf16(rng.standard_normal((wl.n_tokens, c)).astype(np.float32))
    p, blk = util.build_blocks_gpu(wl)
    got = gpu_module(wl, p, blk, wl.k, pe, w, bias, dxc, dx0.reshape(wl.k.shape))
    f = mod.forward(x, pe, w, bias)
    g = mod.backward(x, pe, w, bias, dxc)
    util.assert_close(got["x_cmp"].reshape(-1, c), f.x_cmp, "bf16", "x_cmp")
    util.assert_close(got["dx"].reshape(-1, c), dx0 + g.dx, "bf16", "dx")
    util.assert_close(got["dpe"], g.dpe, "bf16", "dpe")
    util.assert_close(got["dw"], g.dw, "bf16", "dw")
    util.assert_close(got["dbias"], g.dbias, "bf16", "dbias")


def test_module_full_size_g128():
    """The benchmark workload itself (62 229 tokens, C = 128), in the launch configuration ``bench.py --cmp-module``
    times; the fp64 oracle covers every output at this size in seconds."""
    wl = inputs.make_workload("g128")
    orc, mod = module_oracle(wl)
    c = wl.n_heads_kv * wl.head_dim
    pe, w, bias = draw_weights(59, wl.m_cmp, c)
    x = wl.k.reshape(wl.n_tokens, c)
    rng = np.random.default_rng(66)
    dxc = rng.standard_normal((orc.blocks.n_blocks["cmp"], c)).astype(np.float32)
    dx0 = inputs.round_to_bf16(rng.standard_normal((wl.n_tokens, c)).astype(np.float32))
    p, blk = util.build_blocks_gpu(wl)
    got = gpu_module(wl, p, blk, wl.k, pe, w, bias, dxc, dx0.reshape(wl.k.shape))
    f = mod.forward(x, pe, w, bias)
    g = mod.backward(x, pe, w, bias, dxc)
    util.assert_close(got["x_cmp"].reshape(-1, c), f.x_cmp, "bf16", "x_cmp")
    util.assert_close(got["dx"].reshape(-1, c), dx0 + g.dx, "bf16", "dx")
    util.assert_close(got["dpe"], g.dpe, "bf16", "dpe")
    util.assert_close(got["dw"], g.dw, "bf16", "dw")
    util.assert_close(got["dbias"], g.dbias, "bf16", "dbias")


def test_identity_module_equals_plain_pool_bitwise():
    """Centre weight = identity, PE = bias = 0: the module's output is the mean pool; fed to ssa_forward_pooled it
    must give the same result as ssa_forward does with its own pooling (same rounding: fp32 mean -> bf16)."""
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.random_points_workload(56, 32, (1500, 700), 16, 2, 64, (4, 8, 8), 6, "bf16")
    c = 128
    pe = np.zeros((64, c), np.float32)
    w = np.zeros((27, c, c), np.float32)
    w[13] = np.eye(c)
    bias = np.zeros(c, np.float32)
    p, blk = util.build_blocks_gpu(wl)
    kc = gpu_module(wl, p, blk, wl.k, pe, w, bias)["x_cmp"]
    vc = gpu_module(wl, p, blk, wl.v, pe, w, bias)["x_cmp"]
    plain = util.run_gpu(wl, backward=False, blocks=(p, blk))
    q, k, v, g = (util.to_dev(a, "bf16") for a in (wl.q, wl.k, wl.v, wl.gates))
    out = torch.zeros_like(q)
    idx = torch.zeros((wl.n_tokens, 2, 6), dtype=torch.int32, device="cuda")
    ssa.ssa_forward_pooled(p, blk, q, k, v, g, util.to_dev(kc, "bf16"), util.to_dev(vc, "bf16"), out, None, idx, None)
    torch.cuda.synchronize()
    assert np.array_equal(util.to_np(idx), plain.topk_idx)
    assert np.array_equal(util.to_np(out), plain.out)


def test_module_feeds_attention_end_to_end():
    """K and V each go through their own module; the block-level tokens feed the compression branch and the
    selection scores; gradients flow back through ssa_backward_pooled and the module's backward."""
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.random_points_workload(57, 32, (1400, 900), 16, 2, 64, (4, 8, 8), 5, "bf16")
    n, c = wl.n_tokens, 128
    orc, mod = module_oracle(wl)
    wk, wv = draw_weights(571, 4, c), draw_weights(572, 4, c)
    p, blk = util.build_blocks_gpu(wl)
    nc = blk.counts()[0]
    # ---- HIP path
    q, k, v, g, do = (util.to_dev(a, "bf16") for a in (wl.q, wl.k, wl.v, wl.gates, wl.dout))
    dev = lambda ws: tuple(util.to_dev(a, "bf16") for a in ws)
    dwk, dwv = dev(wk), dev(wv)
    kc = torch.empty((nc, 2, 64), dtype=torch.bfloat16, device="cuda")
    vc = torch.empty_like(kc)
    ssa.ssa_compress_forward(p, blk, k, *dwk, kc)
    ssa.ssa_compress_forward(p, blk, v, *dwv, vc)
    out = torch.empty_like(q)
    ob = torch.empty((3,) + tuple(q.shape), dtype=q.dtype, device="cuda")
    lse = torch.empty((3, n, 16), dtype=torch.float32, device="cuda")
    idx = torch.empty((n, 2, 5), dtype=torch.int32, device="cuda")
    ssa.ssa_forward_pooled(p, blk, q, k, v, g, kc, vc, out, lse, idx, ob)
    dq, dk, dv, dg = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v), torch.empty_like(g)
    dkc = torch.empty((nc, 2, 64), dtype=torch.float32, device="cuda")
    dvc = torch.empty_like(dkc)
    ssa.ssa_backward_pooled(p, blk, q, k, v, g, kc, vc, ob, lse, idx, do, dq, dk, dv, dg, dkc, dvc)
    grads = {}
    for name, x, ws, dxc, dx in (("k", k, dwk, dkc, dk), ("v", v, dwv, dvc, dv)):
        dpe = torch.empty((64, c), dtype=torch.float32, device="cuda")
        dw = torch.empty((27, c, c), dtype=torch.float32, device="cuda")
        db = torch.empty((c,), dtype=torch.float32, device="cuda")
        ssa.ssa_compress_backward(p, blk, x, *ws, dxc, dx, dpe, dw, db)
        grads[name] = (util.to_np(dpe), util.to_np(dw), util.to_np(db))
    torch.cuda.synchronize()
    # ---- oracle chain
    fk = mod.forward(wl.k.reshape(n, c), *wk)
    fv = mod.forward(wl.v.reshape(n, c), *wv)
    okc, ovc = fk.x_cmp.reshape(nc, 2, 64), fv.x_cmp.reshape(nc, 2, 64)
    util.assert_close(util.to_np(kc), okc, "bf16", "k_cmp")
    ref_own = orc.forward(wl.q, wl.k, wl.v, wl.gates, want_scores=True, k_cmp=okc, v_cmp=ovc)
    gi = util.to_np(idx)
    util.check_topk(gi, ref_own, orc, "bf16")
    ref = orc.forward(wl.q, wl.k, wl.v, wl.gates, topk_idx=gi, k_cmp=okc, v_cmp=ovc)
    util.assert_close(util.to_np(out), ref.out, "bf16", "out")
    rb = orc.backward(wl.q, wl.k, wl.v, wl.gates, wl.dout, gi, out_branch=ref.out_branch, k_cmp=okc, v_cmp=ovc)
    util.assert_close(util.to_np(dq), rb.dq, "bf16", "dq")
    util.assert_close(util.to_np(dkc), rb.dk_cmp, "bf16", "dk_cmp")
    util.assert_close(util.to_np(dvc), rb.dv_cmp, "bf16", "dv_cmp")
    for name, x, ws, dxc, tok_grad, got_tok in (("k", wl.k, wk, rb.dk_cmp, rb.dk, dk), ("v", wl.v, wv, rb.dv_cmp, rb.dv, dv)):
        gb = mod.backward(x.reshape(n, c), *ws, dxc.reshape(nc, c))
        util.assert_close(util.to_np(got_tok).reshape(n, c), tok_grad.reshape(n, c) + gb.dx, "bf16", "d" + name)
        util.assert_close(grads[name][0], gb.dpe, "bf16", f"dpe_{name}")
        util.assert_close(grads[name][1], gb.dw, "bf16", f"dw_{name}")
        if name == "v":
            util.assert_close(grads[name][2], gb.dbias, "bf16", f"dbias_{name}")
        else:
            # a constant added to every block-level key leaves the softmax unchanged: the exact gradient is zero and
            # what remains is the rounding of its terms, measured against their absolute sum
            assert np.abs(gb.dbias).max() < 1e-9
            assert np.abs(grads[name][2]).max() <= 2e-3 * np.abs(dxc.reshape(nc, c)).sum(axis=0).max()


def test_module_validation():
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.random_points_workload(58, 8, (100,), 4, 2, 16, (2, 4, 4), 2, "f32")
    p, blk = util.build_blocks_gpu(wl)
    assert ssa.ssa_compress_workspace_bytes(p, blk, False) == 0          # fp32: not covered
    x = util.to_dev(wl.k, "f32")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_compress_forward(p, blk, x, x, x, x, x, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -8
    wl2 = inputs.random_points_workload(59, 8, (100,), 4, 2, 16, (2, 4, 4), 2, "bf16")
    p2, blk2 = util.build_blocks_gpu(wl2)
    xb = util.to_dev(wl2.k, "bf16")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_compress_forward(p2, blk2, xb, xb, xb, xb, xb, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -7                                           # workspace too small, nothing launched
    with pytest.raises(ssa.SSAError) as e:                                # pooled attention: fp32 is not covered
        ssa.ssa_forward_pooled(p, blk, x, x, x, x, x, x, x)
    assert e.value.status == -8
