"""GPU: the entry point that allocates nothing (ssa_gate_forward_static, for callers that cannot call hipMalloc) against
the entry point it is a variant of (ssa_gate_forward), through the C ABI.  The two share their kernels, so the results
must be equal bit for bit; both are also held to the fp64 oracle.  Two calls in a row, the second on a smaller input
(fewer tokens, fewer heads, a smaller layer), since every call on a GPU reuses the same static array."""
import numpy as np
import pytest

from oracle.gate import gate_forward
from paper_2505_17412_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu


def _case(seed, n, hq, dm):
    rng = np.random.default_rng(seed)
    r = inputs.round_to_bf16
    j = 3 * hq
    x = r(rng.standard_normal((n, dm)).astype(np.float32))
    w = r((rng.standard_normal((dm, j)) / np.sqrt(dm)).astype(np.float32))
    b = r(rng.standard_normal(j).astype(np.float32))
    return x, w, b


def test_static_scratch_gate_forward_matches_the_allocating_entry_point():
    import torch
    from paper_2505_17412_amd import ssa
    # the larger problem first, then a smaller one in every dimension: stale weights of the first call (rows and
    # columns the second does not overwrite) must not reach the second result
    for seed, n, hq, dm in ((71, 3000, 20, 1024), (72, 517, 4, 256)):
        x, w, b = _case(seed, n, hq, dm)
        p = ssa.make_params(n, 1, 8, 2, 4, 4, 1, hq, hq, 64, "bf16")
        tx, tw, tb = (util.to_dev(a, "bf16") for a in (x, w, b))
        want = torch.full((n, hq, 3), float("nan"), dtype=torch.bfloat16, device="cuda")
        got = torch.full((n, hq, 3), float("nan"), dtype=torch.bfloat16, device="cuda")
        ssa.ssa_gate_forward(p, dm, tx, tw, tb, want)
        ssa.ssa_gate_forward_static(p, dm, tx, tw, tb, got)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (seed, n, hq, dm)
        util.assert_close(util.to_np(got).reshape(n, 3 * hq), gate_forward(x, w, b), "bf16", "gates (static scratch)")


def test_static_scratch_gate_forward_rejects_sizes_beyond_its_array():
    import torch
    from paper_2505_17412_amd import ssa
    p = ssa.make_params(16, 1, 8, 2, 4, 4, 1, 4, 4, 64, "bf16")
    x = torch.zeros((16, 8192), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((8192, 12), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((12,), dtype=torch.bfloat16, device="cuda")
    g = torch.zeros((16, 4, 3), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_gate_forward_static(p, 8192, x, w, b, g)   # the static array holds 64 x 4096 weights
    assert e.value.status == -8
