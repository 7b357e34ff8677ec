"""GPU: the sequence (one-dimensional) partition built by ssa_build_blocks_1d, and the attention path on it, against
the oracle's own sequence partition (pinned on the CPU in test_seq1d_pins.py)."""
import numpy as np
import pytest

from oracle.blocks import build_blocks_1d
from paper_2505_17412_amd import inputs
from tests import util
from tests.test_gpu_parity import full_parity

pytestmark = pytest.mark.gpu

ARRAYS = ("PERM", "INV_PERM", "CMP_START", "SLC_START", "WIN_START", "SLC_CHILD_START", "CMP_BATCH", "SLC_BATCH", "TOK_WIN")


def export_all(blk):
    import torch
    out = {}
    for name in ARRAYS:
        out[name] = blk.export(name.lower()).cpu().numpy()
    torch.cuda.synchronize()
    return out, blk.counts()


@pytest.mark.parametrize("lens,l", [
    ((1500, 0, 64, 513, 4096, 1), (64, 512, 512)),
    ((50, 0, 71), (6, 18, 25)),
    ((70000,), (32, 64, 512)),
    ((0, 0), (2, 4, 4)),
])
def test_sequence_blocks_bit_exact(lens, l):
    wl = inputs.make_sequence_workload(1, lens, l=l, with_tensors=False)
    print("seq blocks", lens, l, flush=True)
    p, blk = util.build_blocks_gpu(wl)
    got, counts = export_all(blk)
    ref = build_blocks_1d(wl.batch_offsets, *l)
    assert counts == (ref.n_blocks["cmp"], ref.n_blocks["slc"], ref.n_blocks["win"])
    expect = dict(PERM=ref.perm, INV_PERM=ref.inv_perm, CMP_START=ref.start["cmp"], SLC_START=ref.start["slc"],
                  WIN_START=ref.start["win"], SLC_CHILD_START=ref.slc_child_start, CMP_BATCH=ref.cmp_batch,
                  SLC_BATCH=ref.slc_batch, TOK_WIN=ref.tok_win)
    for name in ARRAYS:
        assert np.array_equal(got[name], expect[name]), name


def test_sequence_bad_offsets_are_refused():
    import torch
    from paper_2505_17412_amd import ssa
    p = ssa.make_params(100, 2, 0, 4, 8, 8, 2, 4, 2, 16, "f32")
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_build_blocks_1d(p, torch.tensor([0, 60, 90], dtype=torch.int32, device="cuda"))
    assert e.value.status == -5
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_build_blocks_1d(p, torch.tensor([0, 70, 60], dtype=torch.int32, device="cuda"))
    assert e.value.status == -5
    p.m_slc = 6  # not a multiple of m_cmp
    with pytest.raises(ssa.SSAError) as e:
        ssa.ssa_build_blocks_1d(p, torch.tensor([0, 60, 100], dtype=torch.int32, device="cuda"))
    assert e.value.status == -3


@pytest.mark.parametrize("seed,lens,hq,hkv,d,l,topk,dtype", [
    (21, (300, 0, 171), 4, 2, 16, (6, 18, 25), 3, "f32"),          # generic path, ragged block lengths
    (22, (1200, 700), 16, 2, 64, (32, 64, 512), 16, "bf16"),       # the sequence-model block sizes
    (23, (1531,), 16, 1, 64, (16, 64, 128), 8, "bf16"),
    (24, (900, 333), 16, 2, 128, (32, 64, 256), 6, "bf16"),
])
def test_sequence_parity(seed, lens, hq, hkv, d, l, topk, dtype):
    wl = inputs.make_sequence_workload(seed, lens, hq, hkv, d, l, topk, dtype)
    full_parity(wl)


def test_compression_module_refuses_sequences():
    import torch
    from paper_2505_17412_amd import ssa
    wl = inputs.make_sequence_workload(3, (256,), 16, 2, 64, (4, 8, 8), 4, "bf16")
    p, blk = util.build_blocks_gpu(wl)
    assert ssa.ssa_compress_workspace_bytes(p, blk, False) == 0


def test_sequence_full_size_sampled_queries():
    """The 65 536-token sequence that ``bench.py --seq1d`` times, same launch configuration; the oracle visits every
    64th query (dO is zero elsewhere, so dK and dV are comparable in full)."""
    wl = inputs.make_sequence_workload(2001, (65536,))
    full_parity(wl, queries=np.arange(17, wl.n_tokens, 64, dtype=np.int32))
