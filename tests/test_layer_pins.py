"""CPU pin of the layer oracle's backward chain: the directional derivative of sum(dy * y) along a random
perturbation of the input and of every parameter, by central differences of the fp64 forward chain with the selected
sets held fixed, must equal the inner product of the oracle's gradients with that perturbation."""
import numpy as np

from oracle.layer import LayerWeights, layer_backward, layer_forward
from oracle.ssa_oracle import oracle_for
from paper_2505_17412_amd import inputs

FIELDS = ("wq", "wk", "wv", "wg", "bg", "wo", "bq", "bk", "bv", "bo")


def test_layer_gradients_match_central_differences():
    wl = inputs.random_points_workload(31, 8, (37, 20), 4, 2, 8, (2, 4, 4), 3, "f32")
    orc = oracle_for(wl)
    n, hq, hkv, d, dm = wl.n_tokens, 4, 2, 8, 24
    rng = np.random.default_rng(9)
    g = lambda *s: rng.standard_normal(s)
    w = LayerWeights(wq=g(hq * d, dm) / 5, wk=g(hkv * d, dm) / 5, wv=g(hkv * d, dm) / 5, wg=g(dm, 3 * hq) / 5,
                     bg=g(3 * hq), wo=g(dm, hq * d) / 5, bq=g(hq * d) / 5, bk=g(hkv * d) / 5, bv=g(hkv * d) / 5, bo=g(dm))
    x, dy = g(n, dm), g(n, dm)
    f = layer_forward(orc, x, w)
    grads = layer_backward(orc, x, w, f, dy)
    dirs = {nm: g(*getattr(w, nm).shape) for nm in FIELDS}
    dirx = g(n, dm)
    analytic = float(np.sum(grads["dx"] * dirx)) + sum(float(np.sum(grads["d" + nm] * dirs[nm])) for nm in FIELDS)

    def loss(eps):
        w2 = LayerWeights(**{nm: getattr(w, nm) + eps * dirs[nm] for nm in FIELDS})
        return float(np.sum(layer_forward(orc, x + eps * dirx, w2, topk_idx=f.attn.topk_idx).y * dy))

    eps = 1e-5
    numeric = (loss(eps) - loss(-eps)) / (2 * eps)
    assert abs(numeric - analytic) <= 1e-6 * max(abs(analytic), 1.0), (numeric, analytic)
    # each parameter alone: a dropped or swapped term cannot hide behind the others
    for nm in FIELDS + ("x",):
        def loss1(e):
            w2 = LayerWeights(**{k: getattr(w, k) + (e * dirs[k] if k == nm else 0.0) for k in FIELDS})
            return float(np.sum(layer_forward(orc, x + (e * dirx if nm == "x" else 0.0), w2, topk_idx=f.attn.topk_idx).y * dy))
        num = (loss1(eps) - loss1(-eps)) / (2 * eps)
        ana = float(np.sum(grads["dx"] * dirx)) if nm == "x" else float(np.sum(grads["d" + nm] * dirs[nm]))
        assert abs(num - ana) <= 1e-6 * max(abs(ana), 1.0), (nm, num, ana)


def test_layer_with_learned_compression_matches_central_differences():
    """The same pin with the learned compression module in the chain: its six parameter arrays get gradients, and dk,
    dv gain the part that flows back through the module."""
    from oracle.cmp_module import CompressionModule
    wl = inputs.random_points_workload(32, 8, (41, 23), 4, 2, 8, (2, 4, 4), 3, "f32")
    orc = oracle_for(wl)
    b = orc.blocks
    module = CompressionModule(wl.coords, wl.batch_offsets, wl.m_cmp, b.ids["cmp"], b.n_blocks["cmp"])
    n, hq, hkv, d, dm = wl.n_tokens, 4, 2, 8, 16
    c = hkv * d
    rng = np.random.default_rng(10)
    g = lambda *s: rng.standard_normal(s)
    fields = FIELDS + ("pe_k", "wc_k", "bc_k", "pe_v", "wc_v", "bc_v")
    w = LayerWeights(wq=g(hq * d, dm) / 4, wk=g(hkv * d, dm) / 4, wv=g(hkv * d, dm) / 4, wg=g(dm, 3 * hq) / 4,
                     bg=g(3 * hq), wo=g(dm, hq * d) / 5, bq=g(hq * d) / 5, bk=g(hkv * d) / 5, bv=g(hkv * d) / 5, bo=g(dm),
                     pe_k=g(8, c) / 3, wc_k=g(27, c, c) / 6, bc_k=g(c) / 3, pe_v=g(8, c) / 3, wc_v=g(27, c, c) / 6,
                     bc_v=g(c) / 3)
    x, dy = g(n, dm), g(n, dm)
    f = layer_forward(orc, x, w, module=module)
    plain = layer_forward(orc, x, w, topk_idx=f.attn.topk_idx)
    assert np.abs(f.y - plain.y).max() > 1e-3  # the module is in the chain
    grads = layer_backward(orc, x, w, f, dy, module=module)
    dirs = {nm: g(*getattr(w, nm).shape) for nm in fields}
    dirx = g(n, dm)
    eps = 1e-5
    for nm in fields + ("x",):
        def loss1(e):
            w2 = LayerWeights(**{k: getattr(w, k) + (e * dirs[k] if k == nm else 0.0) for k in fields})
            return float(np.sum(layer_forward(orc, x + (e * dirx if nm == "x" else 0.0), w2, topk_idx=f.attn.topk_idx,
                                              module=module).y * dy))
        num = (loss1(eps) - loss1(-eps)) / (2 * eps)
        ana = float(np.sum(grads["dx"] * dirx)) if nm == "x" else float(np.sum(grads["d" + nm] * dirs[nm]))
        assert abs(num - ana) <= 1e-6 * max(abs(ana), 1.0), (nm, num, ana)
