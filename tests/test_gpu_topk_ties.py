"""GPU: the top-k decision of the bf16 matrix-core forward (the path the benchmark runs) on real ties.

With Q = 0 every compression-attention probability of an item is the same number, so the score of a selection block
(eq. (6)) is that number times its count of child compression blocks: the selected set is an integer closed form,
the blocks of the token's item ordered by (child count descending, block id ascending), with many exact ties (the rule
stated after eq. (6): top-k by score; ties to the lowest id).  The expected sets below come from the oracle's block
structure alone (child ranges per selection block, block ranges per item); no score is computed on the CPU.  The
comparison is exact, with no margin.  One case per size class of the search inside the forward kernel (up to 512, up
to 1024 and more than 1024 selection blocks per item), each with an item holding fewer than T blocks (all taken, padded
with -1), for 8 and 16 query heads per KV head and for a small head group.
"""
import numpy as np
import pytest

from oracle import blocks as oblocks
from paper_2505_17412_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu


def closed_form_sets(wl):
    b = oblocks.build_blocks(wl.coords, wl.batch_offsets, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win)
    children = np.diff(b.slc_child_start)
    T = wl.topk
    per_item = []
    for it in range(wl.n_batch):
        s0, s1 = int(b.slc_batch[it]), int(b.slc_batch[it + 1])
        order = sorted(range(s0, s1), key=lambda j: (-int(children[j]), j))[:T]
        row = np.full(T, -1, dtype=np.int32)
        row[: len(order)] = sorted(order)
        per_item.append(row)
    item_of_token = np.searchsorted(wl.batch_offsets, np.arange(wl.n_tokens), side="right") - 1
    return np.stack(per_item)[item_of_token], b


@pytest.mark.parametrize("seed,grid,n,hq,hkv,d,m,topk,lo,hi", [
    (81, 32, (1500, 3, 700), 16, 2, 64, (4, 8, 8), 8, 1, 512),          # <= 512 blocks per item; an item of <= 3 blocks
    (82, 32, (1200, 2), 16, 1, 64, (4, 8, 8), 8, 1, 512),               # 16 query heads on one KV head
    (83, 64, (900, 5), 16, 2, 64, (2, 4, 4), 8, 513, 1024),             # (512, 1024] blocks per item
    (84, 64, (3000, 4), 16, 2, 64, (2, 4, 4), 8, 1025, 4096),           # more than 1024 blocks per item
    (85, 32, (1000, 2), 8, 4, 64, (4, 8, 8), 6, 1, 512),                # 2 query heads per KV head
    (86, 64, (2500,), 16, 2, 128, (2, 4, 4), 16, 1025, 4096),           # head_dim 128, T = 16
])
def test_zero_queries_select_by_child_count_on_the_matrix_core_path(seed, grid, n, hq, hkv, d, m, topk, lo, hi):
    wl = inputs.random_points_workload(seed, grid, n, hq, hkv, d, m, topk, "bf16")
    wl.q[:] = 0
    expect, b = closed_form_sets(wl)
    assert lo <= b.s_max <= hi, b.s_max
    children = np.diff(b.slc_child_start)
    assert len(np.unique(children)) < len(children) // 4   # the closed form really is full of ties
    if len(n) > 1:
        assert int(np.min(np.diff(b.slc_batch))) < topk    # an item with fewer than T blocks
    g = util.run_gpu(wl, backward=False)
    assert np.array_equal(g.topk_idx, np.broadcast_to(expect[:, None, :], g.topk_idx.shape))
