"""Writes tests/golden/tiny_case.json: stored results of the fp64 oracle on one tiny seeded problem.

The paper prints no worked numerical example of SSA (its printed numbers are model-level metrics and the 3.9x / 9.6x
kernel speed-ups of Sec. 4.3, which are context, not values an implementation can be checked against), so the stored
values here are the oracle's own, written by this script, which calls nothing but `oracle/` and the seeded input
generator.  They pin the oracle against accidental change (tests/test_golden.py) and give the HIP path a fixed target
that no run of the HIP path ever produced.

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.ssa_oracle import oracle_for  # noqa: E402
from paper_2505_17412_amd import inputs  # noqa: E402

CASE = dict(seed=7, grid=8, n=(23, 0, 17), hq=4, hkv=2, d=8, m=(2, 4, 4), topk=2, dtype="f32")


def compute():
    c = CASE
    wl = inputs.random_points_workload(c["seed"], c["grid"], c["n"], c["hq"], c["hkv"], c["d"], c["m"], c["topk"], c["dtype"])
    orc = oracle_for(wl)
    f = orc.forward(wl.q, wl.k, wl.v, wl.gates, want_scores=True)
    b = orc.backward(wl.q, wl.k, wl.v, wl.gates, wl.dout, f.topk_idx, out_branch=f.out_branch)
    blk = orc.blocks
    return wl, {
        "case": {k: (list(v) if isinstance(v, tuple) else v) for k, v in c.items()},
        "perm": blk.perm.tolist(),
        "cmp_start": blk.start["cmp"].tolist(), "slc_start": blk.start["slc"].tolist(), "win_start": blk.start["win"].tolist(),
        "slc_child_start": blk.slc_child_start.tolist(), "cmp_batch": blk.cmp_batch.tolist(), "slc_batch": blk.slc_batch.tolist(),
        "topk_idx": f.topk_idx.tolist(),
        "out": np.round(f.out, 12).tolist(),
        "lse": np.round(f.lse, 12).tolist(),
        "dq": np.round(b.dq, 12).tolist(), "dk": np.round(b.dk, 12).tolist(), "dv": np.round(b.dv, 12).tolist(),
        "dgates": np.round(b.dgates, 12).tolist(),
    }


if __name__ == "__main__":
    _, data = compute()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_case.json")
    with open(path, "w") as fh:
        json.dump(data, fh, separators=(",", ":"))
    print("wrote", path, os.path.getsize(path), "bytes")
