"""GPU: the linear projections y = x W^T + b, forward and backward, against the fp64 oracle, element by element
(bf16 tolerances of the attention path: 2e-2 max / 1e-3 mean relative to max|reference|)."""
import numpy as np
import pytest

from oracle.linear import linear_backward, linear_forward
from paper_2505_17412_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,n,d_in,d_out,bias", [
    (71, 1000, 256, 128, True),      # ragged token tail, one feature tile
    (72, 333, 128, 384, False),      # a single contraction chunk pair, three feature tiles
    (73, 1, 128, 128, True),         # a single token
    (74, 4100, 1024, 1024, True),    # the layer's square projection; several token splits in the weight gradient
    (75, 2500, 1024, 128, False),    # the key / value projection of 2 KV heads of 64
    (76, 128, 384, 256, True),       # exactly one token tile
    (77, 62229, 1024, 1024, True),   # the shapes bench.py --linear times
    (78, 62229, 1024, 128, True),
])
def test_linear_forward_backward(seed, n, d_in, d_out, bias):
    import torch
    from paper_2505_17412_amd import ssa
    print("linear", n, d_in, d_out, bias, flush=True)
    rng = np.random.default_rng(seed)
    r = inputs.round_to_bf16
    x = r(rng.standard_normal((n, d_in)).astype(np.float32))
    w = r((rng.standard_normal((d_out, d_in)) / np.sqrt(d_in)).astype(np.float32))
    b = r(rng.standard_normal(d_out).astype(np.float32)) if bias else None
    dy = r(rng.standard_normal((n, d_out)).astype(np.float32))
    tx, tw, tdy = (util.to_dev(a, "bf16") for a in (x, w, dy))
    tb = util.to_dev(b, "bf16") if bias else None
    y = torch.full((n, d_out), float("nan"), dtype=torch.bfloat16, device="cuda")
    ssa.ssa_linear_forward(tx, tw, tb, y)
    torch.cuda.synchronize()
    util.assert_close(util.to_np(y), linear_forward(x, w, b), "bf16", "y")
    dx = torch.full((n, d_in), float("nan"), dtype=torch.bfloat16, device="cuda")
    dw = torch.full((d_out, d_in), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((d_out,), float("nan"), dtype=torch.float32, device="cuda") if bias else None
    ssa.ssa_linear_backward(tx, tw, tdy, dx, dw, db)
    torch.cuda.synchronize()
    rdx, rdw, rdb = linear_backward(x, w, dy)
    util.assert_close(util.to_np(dx), rdx, "bf16", "dx")
    # the parameter gradients are fp32 sums of exact bf16 products: far inside the bf16 tolerance
    util.assert_close(util.to_np(dw), rdw, "bf16", "dw", scale=0.01)
    if bias:
        util.assert_close(util.to_np(db), rdb, "bf16", "dbias", scale=0.01)
    # without dx: the parameter gradients alone, bit-identical to the first call
    dw2 = torch.full_like(dw, float("nan"))
    ssa.ssa_linear_backward(tx, tw, tdy, None, dw2, None)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw2)


def test_linear_validation_and_empty():
    import torch
    from paper_2505_17412_amd import ssa
    assert ssa.ssa_linear_workspace_bytes(10, 100, 128, True) == 0            # d_in not a multiple of 128
    x = torch.zeros((10, 128), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((128, 128), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((10, 128), dtype=torch.bfloat16, device="cuda")
    bad = torch.zeros((10, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_linear_forward(bad, torch.zeros((128, 96), dtype=torch.bfloat16, device="cuda"), None, y)
    assert e.value.status == -8
    dw = torch.full((128, 128), float("nan"), dtype=torch.float32, device="cuda")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_linear_backward(x, w, y, None, dw, None, workspace=torch.empty(8, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -7
    # no tokens: nothing to write forward, zero parameter gradients backward
    e0 = torch.zeros((0, 128), dtype=torch.bfloat16, device="cuda")
    ssa.ssa_linear_forward(e0, w, None, e0)
    db = torch.full((128,), float("nan"), dtype=torch.float32, device="cuda")
    ssa.ssa_linear_backward(e0, w, e0, e0, dw, db)
    torch.cuda.synchronize()
    assert float(dw.abs().max()) == 0.0 and float(db.abs().max()) == 0.0
