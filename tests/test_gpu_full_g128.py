"""GPU: EVERY query of the benchmark workload against the oracle, forward and backward.

Config "g128" (128^3 grid, ~62k tokens, bf16, 16 query / 2 KV heads of 64, top-16) in the launch configuration
bench.py times.  The query set is cut into eight interleaved slices (query t belongs to slice t mod 8), one test case
each, so that no case keeps the oracle busy for more than about half a minute; together the cases cover all tokens.
Forward: out, the three branch outputs and log-sum-exps, and the selected sets (two-level contract of the other parity
tests) for the slice's queries.  Backward: dO is zero outside the slice (the backward pass is linear in dO and rows with
dO = 0 contribute nothing), so dQ and dgates are compared on the slice and dK, dV in full.  The error figures and the
number of rows whose selected set differs from the oracle's are printed per slice.
"""
import functools

import numpy as np
import pytest

from oracle.ssa_oracle import oracle_for
from paper_2505_17412_amd import harness, inputs
from tests import util

pytestmark = pytest.mark.gpu

N_SLICES = 8


@functools.lru_cache(maxsize=1)
def _shared():
    wl = inputs.make_workload("g128")
    blocks = harness.build_blocks_gpu(wl)
    fwd = harness.run_gpu(wl, backward=False, blocks=blocks)
    return wl, blocks, fwd, oracle_for(wl)


@pytest.mark.parametrize("k", range(N_SLICES))
def test_g128_every_query_forward_backward(k):
    wl, blocks, fwd, orc = _shared()
    queries = np.arange(k, wl.n_tokens, N_SLICES, dtype=np.int32)
    dout = np.zeros_like(wl.dout)
    dout[queries] = wl.dout[queries]
    g = harness.run_gpu(wl, backward=True, dout=dout, blocks=blocks)
    assert np.array_equal(g.topk_idx, fwd.topk_idx) and np.array_equal(g.out, fwd.out)  # same forward every time
    ref_own = orc.forward(wl.q, wl.k, wl.v, wl.gates, queries=queries, want_scores=True)
    ndiff = util.check_topk(g.topk_idx, ref_own, orc, wl.dtype, queries=queries)
    ref = orc.forward(wl.q, wl.k, wl.v, wl.gates, queries=queries, topk_idx=g.topk_idx)
    errs = {"out": util.assert_close(g.out[queries], ref.out[queries], wl.dtype, "out")}
    for b, nm in enumerate(("cmp", "slc", "win")):
        errs["out_" + nm] = util.assert_close(g.out_branch[b][queries], ref.out_branch[b][queries], wl.dtype, "out_" + nm)
        errs["lse_" + nm] = util.assert_close(g.lse[b][queries], ref.lse[b][queries], wl.dtype, "lse_" + nm)
    rb = orc.backward(wl.q, wl.k, wl.v, wl.gates, dout, g.topk_idx, out_branch=ref.out_branch, queries=queries)
    errs["dq"] = util.assert_close(g.dq[queries], rb.dq[queries], wl.dtype, "dq")
    errs["dk"] = util.assert_close(g.dk, rb.dk, wl.dtype, "dk")
    errs["dv"] = util.assert_close(g.dv, rb.dv, wl.dtype, "dv")
    errs["dgates"] = util.assert_close(g.dgates[queries], rb.dgates[queries], wl.dtype, "dgates")
    print(f"g128 slice {k}/{N_SLICES}: {len(queries)} queries, selected sets differing from the oracle's (inside the margin): "
          f"{ndiff} of {len(queries) * wl.n_heads_kv} rows; max/mean errors relative to max|ref|: "
          + ", ".join(f"{nm} {e[0]:.1e}/{e[1]:.1e}" for nm, e in errs.items()), flush=True)
