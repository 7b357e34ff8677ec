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
