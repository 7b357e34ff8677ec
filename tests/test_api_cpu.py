"""CPU-only checks of the boundary: the library loads, exports what the header declares, and rejects bad
arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2505_17412_amd import ssa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ssa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ssa_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ssa.lib()
    names = declared_functions()
    assert set(names) == set(ssa.EXPORTED_SYMBOLS)
    for n in names:
        assert getattr(L, n) is not None


def test_error_strings():
    assert ssa.error_string(0) == "ok"
    seen = {ssa.error_string(-i) for i in range(1, 12)}
    assert len(seen) == 11 and "unknown status" not in seen
    assert ssa.error_string(-99) == "unknown status"


@pytest.mark.parametrize("kw,status", [
    (dict(n_tokens=-1), -2), (dict(n_batch=0), -2), (dict(grid=0), -2), (dict(grid=2048), -2),
    (dict(m_cmp=8, m_slc=8), -3), (dict(m_cmp=4, m_slc=2), -3), (dict(m_cmp=0), -3),
    (dict(m_cmp=3, m_slc=6), -8), (dict(m_win=6), -8),
])
def test_build_blocks_rejects_bad_params_before_any_launch(kw, status):
    base = dict(n_tokens=8, n_batch=1, grid=32, m_cmp=4, m_slc=8, m_win=8, topk=4, n_heads_q=4, n_heads_kv=2,
                head_dim=32, dtype="f32")
    base.update(kw)
    p = ssa.make_params(**base)
    h = C.c_void_p()
    # non-NULL dummy pointers: validation must fail before they are used
    rc = ssa.lib().ssa_build_blocks(C.byref(p), 0x1000, 0x1000, None, C.byref(h))
    assert rc == status and h.value is None


def test_null_arguments():
    L = ssa.lib()
    p = ssa.make_params(8, 1, 32, 4, 8, 8, 4, 4, 2, 32, "f32")
    h = C.c_void_p()
    assert L.ssa_build_blocks(None, None, None, None, C.byref(h)) == -1
    assert L.ssa_build_blocks(C.byref(p), None, None, None, C.byref(h)) == -1
    assert L.ssa_forward(C.byref(p), None, *([None] * 8), None, 0, None) == -1
    assert L.ssa_backward(C.byref(p), None, *([None] * 12), None, 0, None) == -1
    assert L.ssa_topk_from_scores(C.byref(p), None, None, None, None) == -1
    assert L.ssa_workspace_bytes(C.byref(p), None, 0) == 0
    assert L.ssa_blocks_counts(None, None, None, None) == -1
    L.ssa_blocks_destroy(None)  # allowed


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: `bench.py --gpus N` with N > 1 exits with a message, before touching the GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
