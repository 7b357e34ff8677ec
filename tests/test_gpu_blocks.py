"""GPU: ssa_build_blocks must reproduce the oracle's block structure bit for bit (sort + array C, Algorithm 1)."""
import ctypes as C

import numpy as np
import pytest

from oracle.blocks import build_blocks
from oracle.compare import check_block_arrays
from paper_2505_17412_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu

ARRS = ("perm", "inv_perm", "cmp_start", "slc_start", "win_start", "slc_child_start", "cmp_batch", "slc_batch", "tok_win")


def check(wl):
    p, blk = util.build_blocks_gpu(wl)
    ref = build_blocks(wl.coords, wl.batch_offsets, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win)
    assert blk.counts() == (ref.n_blocks["cmp"], ref.n_blocks["slc"], ref.n_blocks["win"])
    assert blk.max_slc_per_item() == ref.s_max
    expect = dict(perm=ref.perm, inv_perm=ref.inv_perm, cmp_start=ref.start["cmp"], slc_start=ref.start["slc"],
                  win_start=ref.start["win"], slc_child_start=ref.slc_child_start, cmp_batch=ref.cmp_batch,
                  slc_batch=ref.slc_batch, tok_win=ref.tok_win)
    exported = {}
    for name in ARRS:
        got = blk.export(name).cpu().numpy()
        assert got.dtype == np.int32 and np.array_equal(got, expect[name]), name
        exported[name] = got
    check_block_arrays(exported, wl.n_tokens, wl.n_batch)  # every index a kernel follows stays in bounds
    blk.destroy()


@pytest.mark.parametrize("name", ["tiny", "g64", "g128", "g128_thick"])
def test_named_workloads(name):
    print("build_blocks", name, flush=True)
    check(inputs.make_workload(name, with_tensors=False))


def test_batch_of_four_shapes():
    check(inputs.make_batch_workload(with_tensors=False))


@pytest.mark.parametrize("seed,grid,n,m,dup", [
    (1, 16, (90, 0, 70), (2, 4, 8), False), (2, 4, (200,), (1, 2, 4), True), (3, 1024, (5000, 1), (4, 8, 16), False),
    (4, 8, (1,), (2, 4, 2), False), (5, 64, (300, 300, 300, 300, 300), (4, 8, 4), True), (6, 32, (0, 0, 257), (4, 8, 8), False),
])
def test_random_points(seed, grid, n, m, dup):
    check(inputs.random_points_workload(seed, grid, n, 2, 1, 8, m, 2, allow_duplicates=dup))


def test_empty_problem():
    wl = inputs.random_points_workload(1, 8, (0, 0), 2, 1, 8, (2, 4, 4), 2)
    p, blk = util.build_blocks_gpu(wl)
    assert blk.counts() == (0, 0, 0)
    blk.destroy()


def test_device_side_errors():
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.random_points_workload(1, 8, (20, 20), 2, 1, 8, (2, 4, 4), 2)
    p = util.params_of(wl)
    bad = wl.coords.copy()
    bad[7, 1] = 8
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_build_blocks(p, torch.from_numpy(bad).cuda(), torch.from_numpy(wl.batch_offsets).cuda())
    assert e.value.status == -6
    bad[7, 1] = -1
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_build_blocks(p, torch.from_numpy(bad).cuda(), torch.from_numpy(wl.batch_offsets).cuda())
    assert e.value.status == -6
    for offs in ([0, 25, 20], [1, 20, 40], [0, 20, 39]):
        with pytest.raises(ssa.SSAError) as e:
            ssa.ssa_build_blocks(p, torch.from_numpy(wl.coords).cuda(), torch.tensor(offs, dtype=torch.int32).cuda())
        assert e.value.status == -5
    # a good call still works afterwards
    blk = ssa.ssa_build_blocks(p, torch.from_numpy(wl.coords).cuda(), torch.from_numpy(wl.batch_offsets).cuda())
    assert blk.counts()[0] > 0


def test_deterministic():
    wl = inputs.make_workload("g64", with_tensors=False)
    a = util.build_blocks_gpu(wl)[1]
    b = util.build_blocks_gpu(wl)[1]
    for name in ARRS:
        assert np.array_equal(a.export(name).cpu().numpy(), b.export(name).cpu().numpy())
