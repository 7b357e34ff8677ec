"""The stored oracle results of tests/golden/tiny_case.json: the oracle must still produce them (CPU), and the HIP
path must match them (GPU) -- a fixed target that no run of the HIP path ever wrote."""
import importlib.util
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _load():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(HERE, "golden", "tiny_case.json")) as fh:
        return mod, json.load(fh)


def test_oracle_reproduces_the_stored_values():
    mod, gold = _load()
    _, now = mod.compute()
    for key in ("perm", "cmp_start", "slc_start", "win_start", "slc_child_start", "cmp_batch", "slc_batch", "topk_idx"):
        assert now[key] == gold[key], key
    for key in ("out", "lse", "dq", "dk", "dv", "dgates"):
        assert np.allclose(np.array(now[key]), np.array(gold[key]), rtol=0, atol=1e-10), key


@pytest.mark.gpu
def test_hip_path_matches_the_stored_values():
    from tests import util
    mod, gold = _load()
    wl, _ = mod.compute()
    p, blk = util.build_blocks_gpu(wl)
    for key in ("perm", "cmp_start", "slc_start", "win_start", "slc_child_start", "cmp_batch", "slc_batch"):
        assert blk.export(key).cpu().numpy().tolist() == gold[key], key
    g = util.run_gpu(wl, blocks=(p, blk))
    assert g.topk_idx.tolist() == gold["topk_idx"]
    util.assert_close(g.out, np.array(gold["out"]), "f32", "out")
    util.assert_close(g.lse, np.array(gold["lse"]), "f32", "lse")
    for key in ("dq", "dk", "dv", "dgates"):
        util.assert_close(getattr(g, key), np.array(gold[key]), "f32", key)
