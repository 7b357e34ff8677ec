"""GPU: a seeded sweep of mid-size problems with randomly drawn shapes (4096-14000 tokens, where the selection
kernels walk their own token order): voxel grids and sequences, 1/2/4 KV heads of 8 or 16 query heads, head
dimensions 32/64/128, top-k 2-32, several block-size triples; forward and backward on every 29th query against the
oracle, to the tolerances of the other parity tests."""
import numpy as np
import pytest

from paper_2505_17412_amd import inputs
from tests.test_gpu_parity import full_parity

pytestmark = pytest.mark.gpu

N_CASES = 12


def draw_case(rng):
    while True:
        hkv, hs, d = int(rng.choice([1, 2, 4])), int(rng.choice([8, 16])), int(rng.choice([32, 64, 128]))
        topk, seed = int(rng.choice([2, 4, 8, 16, 32])), int(rng.integers(1, 1 << 20))
        if rng.random() < 0.6:
            grid = int(rng.choice([32, 64]))
            m = [(4, 8, 8), (2, 4, 8), (4, 8, 16), (2, 8, 8)][int(rng.integers(0, 4))]
            nb = int(rng.integers(1, 4))
            n = tuple(int(x) for x in rng.integers(0, 12000 // nb + 2000, size=nb))
            if sum(n) < 4096 or max(n) > grid ** 3 // 2:
                continue
            return inputs.random_points_workload(seed, grid, n, hkv * hs, hkv, d, m, topk, "bf16")
        lens = tuple(int(x) for x in rng.integers(0, 9000, size=int(rng.integers(1, 4))))
        if sum(lens) < 4096:
            continue
        lc = int(rng.choice([8, 16, 32]))
        l = (lc, lc * int(rng.choice([2, 4])), int(rng.choice([64, 100, 256, 512])))
        return inputs.make_sequence_workload(seed, lens, hkv * hs, hkv, d, l, topk, "bf16")


def test_seeded_sweep_of_mid_size_problems():
    rng = np.random.default_rng(20250517)
    for case in range(N_CASES):
        wl = draw_case(rng)
        print("sweep case", case, wl.name, wl.dims, wl.n_tokens, (wl.m_cmp, wl.m_slc, wl.m_win), wl.topk, flush=True)
        full_parity(wl, queries=np.arange(case % 5, wl.n_tokens, 29, dtype=np.int32))
