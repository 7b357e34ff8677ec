"""GPU: gate predictor sigmoid(x W + b), forward and backward, against the fp64 oracle, element by element
(bf16 tolerances of the attention path: 2e-2 max / 1e-3 mean relative to max|reference|)."""
import numpy as np
import pytest

from oracle.gate import gate_backward, gate_forward
from paper_2505_17412_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,n,hq,dm", [
    (61, 1000, 16, 1024),     # the benchmark's layer: 16 heads of 64
    (62, 77, 4, 128),         # J = 12: one partly filled block of 16 gate columns; ragged token tail
    (63, 2049, 20, 256),      # J = 60
    (64, 1, 8, 128),          # a single token
    (65, 62229, 16, 1024),    # the token count and layer shape bench.py --gate times
])
def test_gate_forward_backward(seed, n, hq, dm):
    import torch
    from paper_2505_17412_amd import ssa
    rng = np.random.default_rng(seed)
    r = inputs.round_to_bf16
    j = 3 * hq
    x = r(rng.standard_normal((n, dm)).astype(np.float32))
    w = r((rng.standard_normal((dm, j)) / np.sqrt(dm)).astype(np.float32))
    b = r(rng.standard_normal(j).astype(np.float32))
    dg = r(rng.standard_normal((n, hq, 3)).astype(np.float32))
    dx0 = r(rng.standard_normal((n, dm)).astype(np.float32))
    p = ssa.make_params(n, 1, 8, 2, 4, 4, 1, hq, hq, dm // hq if dm // hq in (32, 64, 128) else 64, "bf16")
    tx, tw, tb, tdg = (util.to_dev(a, "bf16") for a in (x, w, b, dg))
    gates = torch.full((n, hq, 3), float("nan"), dtype=torch.bfloat16, device="cuda")
    ssa.ssa_gate_forward(p, dm, tx, tw, tb, gates)
    torch.cuda.synchronize()
    ref = gate_forward(x, w, b)
    util.assert_close(util.to_np(gates).reshape(n, j), ref, "bf16", "gates")
    # backward from the oracle's gates rounded to bf16 (the tensor a training step would hold), on both sides
    g16 = r(ref.astype(np.float32))
    dxa = util.to_dev(dx0, "bf16")
    dw = torch.full((dm, j), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((j,), float("nan"), dtype=torch.float32, device="cuda")
    ssa.ssa_gate_backward(p, dm, tx, tw, util.to_dev(g16.reshape(n, hq, 3), "bf16"), tdg, dxa, dw, db)
    torch.cuda.synchronize()
    rdx, rdw, rdb = gate_backward(x, w, g16, dg.reshape(n, j))
    util.assert_close(util.to_np(dxa), dx0 + rdx, "bf16", "dx")
    util.assert_close(util.to_np(dw), rdw, "bf16", "dw")
    util.assert_close(util.to_np(db), rdb, "bf16", "dbias")


def test_gate_validation():
    import torch
    from paper_2505_17412_amd import ssa
    p = ssa.make_params(10, 1, 8, 2, 4, 4, 1, 4, 4, 32, "bf16")
    assert ssa.ssa_gate_workspace_bytes(p, 100, False) == 0                 # d_model not a multiple of 128
    x = torch.zeros((10, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_gate_forward(p, 100, x, x, x, x, workspace=x)
    assert e.value.status == -8
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_gate_forward(p, 128, x, x, x, x, workspace=torch.empty(8, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -7
    pf = ssa.make_params(10, 1, 8, 2, 4, 4, 1, 4, 4, 32, "f32")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_gate_forward(pf, 128, x, x, x, x, workspace=x)
    assert e.value.status == -8
    p0 = ssa.make_params(0, 1, 8, 2, 4, 4, 1, 4, 4, 32, "bf16")
    ssa.ssa_gate_forward(p0, 128, None, None, None, None, workspace=x)       # no tokens: nothing to do
