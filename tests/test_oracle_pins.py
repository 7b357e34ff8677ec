"""CPU-only pins of the fp64 oracle against facts the paper and the mathematics fix.

Each test names the passage it leans on.  The dense reference used below (``dense_attention``) is plain
numpy softmax attention, eq. (2)-(3) of the paper, written here and shared with nothing.
"""
import numpy as np
import pytest

from oracle import brute
from oracle.blocks import build_blocks, morton3
from oracle.ssa_oracle import Oracle, oracle_for
from paper_2505_17412_amd import inputs


def dense_attention(q, k, v, hs, scale):
    """eq. (2)-(3): o_t = sum_i p_ti v_i / sum_j p_tj, p = exp(q.k/sqrt(d)); GQA head h uses KV head h//hs."""
    n, hq, d = q.shape
    o = np.zeros((n, hq, d))
    lse = np.zeros((n, hq))
    for h in range(hq):
        s = (q[:, h] @ k[:, h // hs].T) * scale
        p = np.exp(s)
        o[:, h] = (p @ v[:, h // hs]) / p.sum(axis=1, keepdims=True)
        lse[:, h] = np.log(p.sum(axis=1))
    return o, lse


def small(seed=3, grid=16, n=(70,), hq=4, hkv=2, d=8, m=(2, 4, 4), topk=3, dup=False):
    return inputs.random_points_workload(seed, grid, n, hq, hkv, d, m, topk, "f32", allow_duplicates=dup)


def per_item(wl):
    for b in range(wl.n_batch):
        yield slice(int(wl.batch_offsets[b]), int(wl.batch_offsets[b + 1]))


# ---- P1: top-k >= number of selection blocks  =>  selection branch == dense attention (Algorithm 1 key set)
def test_select_all_blocks_is_dense():
    wl = small(n=(60, 45), topk=64)
    orc = oracle_for(wl)
    r = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    for sl in per_item(wl):
        o, lse = dense_attention(wl.q[sl].astype(float), wl.k[sl].astype(float), wl.v[sl].astype(float), 2, orc.scale)
        np.testing.assert_allclose(r.out_branch[1][sl], o, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(r.lse[1][sl], lse, rtol=1e-11, atol=1e-12)
    # fewer blocks than T: all taken, rest padded with -1
    nblk = np.diff(orc.blocks.slc_batch)
    for b, sl in enumerate(per_item(wl)):
        row = r.topk_idx[sl][0, 0]
        assert np.array_equal(row[:nblk[b]], np.arange(orc.blocks.slc_batch[b], orc.blocks.slc_batch[b + 1]))
        assert np.all(row[nblk[b]:] == -1)


# ---- P2: a window covering the whole grid  =>  window branch == dense attention (window paragraph)
def test_whole_grid_window_is_dense():
    wl = small(n=(50, 33), m=(2, 4, 16))
    orc = oracle_for(wl)
    r = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    for sl in per_item(wl):
        o, lse = dense_attention(wl.q[sl].astype(float), wl.k[sl].astype(float), wl.v[sl].astype(float), 2, orc.scale)
        np.testing.assert_allclose(r.out_branch[2][sl], o, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(r.lse[2][sl], lse, rtol=1e-11, atol=1e-12)


# ---- P3: m_cmp = 1 with distinct voxels  =>  pooled K,V are K,V  =>  compression branch == dense (eq. (5))
def test_unit_compression_block_is_dense():
    wl = small(n=(40, 40), m=(1, 4, 4))
    orc = oracle_for(wl)
    r = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    np.testing.assert_allclose(r.k_cmp, wl.k[orc.blocks.perm], rtol=0, atol=0)
    for sl in per_item(wl):
        o, lse = dense_attention(wl.q[sl].astype(float), wl.k[sl].astype(float), wl.v[sl].astype(float), 2, orc.scale)
        np.testing.assert_allclose(r.out_branch[0][sl], o, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(r.lse[0][sl], lse, rtol=1e-11, atol=1e-12)


# ---- P4: eq. (4) is a gate-weighted SUM of independently normalised branches
def test_gate_combination():
    wl = small(n=(48,), m=(1, 4, 16), topk=64)
    orc = oracle_for(wl)
    g = np.zeros_like(wl.gates, dtype=float)
    g[..., 0], g[..., 1], g[..., 2] = 0.3, 0.9, 0.45
    r = orc.forward(wl.q, wl.k, wl.v, g)
    o, _ = dense_attention(wl.q.astype(float), wl.k.astype(float), wl.v.astype(float), 2, orc.scale)
    np.testing.assert_allclose(r.out, (0.3 + 0.9 + 0.45) * o, rtol=1e-11, atol=1e-12)
    wl2 = small(n=(48,))
    orc2 = oracle_for(wl2)
    base = orc2.forward(wl2.q, wl2.k, wl2.v, wl2.gates)
    for b in range(3):
        onehot = np.zeros_like(wl2.gates, dtype=float)
        onehot[..., b] = 1.0
        rb = orc2.forward(wl2.q, wl2.k, wl2.v, onehot)
        np.testing.assert_allclose(rb.out, base.out_branch[b], rtol=0, atol=0)
    np.testing.assert_allclose(base.out, np.einsum("nhb,bnhd->nhd", wl2.gates.astype(float), base.out_branch),
                               rtol=1e-13, atol=1e-14)


# ---- P5: shuffling the tokens of each item permutes outputs/gradients and leaves the selected sets alone
def test_permutation_equivariance():
    wl = small(n=(55, 37))
    orc = oracle_for(wl)
    f = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    b = orc.backward(wl.q, wl.k, wl.v, wl.gates, wl.dout, f.topk_idx)
    rng = np.random.default_rng(11)
    sh = np.concatenate([o.start + rng.permutation(o.stop - o.start) for o in per_item(wl)])
    orc2 = Oracle(wl.coords[sh], wl.batch_offsets, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win, wl.topk, 4, 2, 8)
    f2 = orc2.forward(wl.q[sh], wl.k[sh], wl.v[sh], wl.gates[sh])
    b2 = orc2.backward(wl.q[sh], wl.k[sh], wl.v[sh], wl.gates[sh], wl.dout[sh], f2.topk_idx)
    assert np.array_equal(f2.topk_idx, f.topk_idx[sh])
    np.testing.assert_allclose(f2.out, f.out[sh], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f2.lse, f.lse[:, sh], rtol=1e-12, atol=1e-13)
    for a2, a in ((b2.dq, b.dq), (b2.dk, b.dk), (b2.dv, b.dv), (b2.dgates, b.dgates)):
        np.testing.assert_allclose(a2, a[sh], rtol=1e-10, atol=1e-12)


# ---- P6: brute force with explicit N x N masks on tiny inputs (second, independent route)
@pytest.mark.parametrize("seed,n,m,topk,hq,hkv", [(1, (40,), (2, 4, 4), 2, 4, 2), (2, (30, 26), (2, 4, 8), 3, 4, 1),
                                                   (5, (50,), (1, 2, 4), 5, 2, 2), (7, (21, 9, 30), (4, 8, 2), 1, 6, 2)])
def test_brute_force(seed, n, m, topk, hq, hkv):
    wl = inputs.random_points_workload(seed, 8 if max(m) <= 4 else 16, n, hq, hkv, 8, m, topk, "f32")
    orc = oracle_for(wl)
    r = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    bf = brute.brute_forward(wl.coords, wl.batch_offsets, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win, wl.topk,
                             wl.q, wl.k, wl.v, wl.gates)
    assert np.array_equal(r.topk_idx, bf["topk_idx"])
    # pooled keys are listed per block id: compare through the token -> block map
    np.testing.assert_allclose(r.k_cmp, bf["k_cmp"], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(r.out_branch, bf["out_branch"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(r.lse, bf["lse"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(r.out, bf["out"], rtol=1e-10, atol=1e-12)


def test_brute_force_duplicate_voxels():
    wl = small(seed=9, grid=4, n=(40,), m=(1, 2, 2), topk=2, dup=True)  # 40 tokens in 64 cells: duplicates
    assert len({tuple(c) for c in wl.coords}) < 40
    orc = oracle_for(wl)
    r = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    bf = brute.brute_forward(wl.coords, wl.batch_offsets, wl.grid, 1, 2, 2, 2, wl.q, wl.k, wl.v, wl.gates)
    assert np.array_equal(r.topk_idx, bf["topk_idx"])
    np.testing.assert_allclose(r.out, bf["out"], rtol=1e-10, atol=1e-12)


# ---- P7: all V rows equal to one vector c  =>  every branch returns c  =>  out = (sum of gates) * c
def test_constant_values():
    wl = small(n=(64, 20))
    c = np.linspace(-1, 2, 8)
    v = np.broadcast_to(c, wl.v.shape).copy()
    r = oracle_for(wl).forward(wl.q, wl.k, v, wl.gates)
    for b in range(3):
        np.testing.assert_allclose(r.out_branch[b], np.broadcast_to(c, r.out.shape), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r.out, wl.gates.astype(float).sum(-1, keepdims=True) * c, rtol=1e-12, atol=1e-13)


# ---- P8: Q = 0  =>  uniform compression probabilities  =>  score(b) = h_s * children(b) / N_c(item):
#          the selected set is the integer closed form "most children first, ties to the lowest id" (eq. (6))
def test_zero_query_closed_form_selection():
    wl = inputs.make_workload("tiny", topk=6)
    orc = oracle_for(wl)
    b = orc.blocks
    q0 = np.zeros_like(wl.q)
    sub = np.arange(0, wl.n_tokens, 37, dtype=np.int32)
    r = orc.forward(q0, wl.k, wl.v, wl.gates, queries=sub, want_scores=True)
    children = np.diff(b.slc_child_start)
    assert len(set(children.tolist())) > 1 and np.max(np.bincount(children)) > 6  # real ties are present
    order = sorted(range(b.n_blocks["slc"]), key=lambda j: (-int(children[j]), j))[:6]
    expect = np.array(sorted(order), dtype=np.int32)
    for t in sub:
        for g in range(wl.n_heads_kv):
            assert np.array_equal(r.topk_idx[t, g], expect)
    hs = wl.n_heads_q // wl.n_heads_kv
    np.testing.assert_allclose(r.scores[sub[0], 0, :b.n_blocks["slc"]], hs * children / b.n_blocks["cmp"], rtol=1e-6)
    # scores of one row sum to h_s (each head's probabilities sum to one)
    np.testing.assert_allclose(r.scores[sub].sum(-1), hs, rtol=1e-5)


def test_topk_tie_break_and_padding():
    orc = oracle_for(small(n=(30, 30), topk=3))
    s = np.zeros((orc.N, orc.Hkv, orc.s_max), dtype=np.float32)
    s[:, :, :] = 1.0
    s[:, 0, 2] = 2.0
    idx = orc.topk_from_scores(s)
    base = orc.blocks.slc_batch[:-1][orc.blocks.tok_item]
    nv = np.diff(orc.blocks.slc_batch)[orc.blocks.tok_item]
    for t in (0, orc.N - 1):
        assert nv[t] >= 4
        assert np.array_equal(idx[t, 0], base[t] + np.array([0, 1, 2]))  # 2 (best), then ties -> 0,1
        assert np.array_equal(idx[t, 1], base[t] + np.array([0, 1, 2]))


# ---- P9: block-aligned translation changes nothing; items of a batch do not see each other
def test_translation_and_batch_isolation():
    wl = small(grid=32, n=(60, 44), m=(2, 4, 8))
    wl.coords[:] = wl.coords % 16  # leave room to translate
    orc = oracle_for(wl)
    f = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    shifted = wl.coords + np.array([8, 16, 8], dtype=np.int32)
    f2 = Oracle(shifted, wl.batch_offsets, 32, 2, 4, 8, wl.topk, 4, 2, 8).forward(wl.q, wl.k, wl.v, wl.gates)
    np.testing.assert_allclose(f2.out, f.out, rtol=1e-12, atol=1e-13)
    # selected sets are the same blocks; ids may be renumbered by the translation only if Morton order changes,
    # which an aligned shift inside the same octant layout does not do for the *set of member tokens*:
    for t in range(0, wl.n_tokens, 9):
        a = {tuple(x) for j in f.topk_idx[t, 0] if j >= 0 for x in wl.coords[orc.blocks.ids["slc"] == j].tolist()}
        ids2 = build_blocks(shifted, wl.batch_offsets, 32, 2, 4, 8).ids["slc"]
        bb = {tuple((np.array(x) - [8, 16, 8]).tolist()) for j in f2.topk_idx[t, 0] if j >= 0
              for x in shifted[(ids2 == j)].tolist()}
        assert a == bb
    for b, sl in enumerate(per_item(wl)):
        off = np.array([0, sl.stop - sl.start], dtype=np.int32)
        alone = Oracle(wl.coords[sl], off, 32, 2, 4, 8, wl.topk, 4, 2, 8).forward(wl.q[sl], wl.k[sl], wl.v[sl], wl.gates[sl])
        np.testing.assert_allclose(alone.out, f.out[sl], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(alone.lse, f.lse[:, sl], rtol=1e-12, atol=1e-13)


# ---- P10: lse is the log-sum-exp of the branch's scaled logits (Algorithm 1's l, read as a running lse)
def test_lse_definition():
    wl = small(n=(52,))
    orc = oracle_for(wl)
    r = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    b = orc.blocks
    t, h = 17, 3
    g = h // 2
    qv = wl.q[t, h].astype(float)
    win = np.where(b.ids["win"] == b.ids["win"][t])[0]
    sel = np.where(np.isin(b.ids["slc"], r.topk_idx[t, g][r.topk_idx[t, g] >= 0]))[0]
    for br, keys in ((1, sel), (2, win)):
        s = (wl.k[keys, g].astype(float) @ qv) * orc.scale
        assert abs(np.log(np.exp(s).sum()) - r.lse[br, t, h]) < 1e-12
    s = (r.k_cmp[:, g] @ qv) * orc.scale
    assert abs(np.log(np.exp(s).sum()) - r.lse[0, t, h]) < 1e-12


# ---- P11: backward == central finite differences of L = sum(dO * O) with the selected sets frozen
def test_backward_finite_differences():
    wl = small(seed=21, n=(36, 22), d=8, m=(2, 4, 4), topk=2)
    orc = oracle_for(wl)
    q, k, v, g, do = (a.astype(np.float64) for a in (wl.q, wl.k, wl.v, wl.gates, wl.dout))
    f = orc.forward(q, k, v, g)
    bw = orc.backward(q, k, v, g, do, f.topk_idx)

    def loss(q_, k_, v_, g_):
        return float((orc.forward(q_, k_, v_, g_, topk_idx=f.topk_idx).out * do).sum())

    rng = np.random.default_rng(5)
    eps = 1e-5
    for name, arr, grad in (("q", q, bw.dq), ("k", k, bw.dk), ("v", v, bw.dv), ("gates", g, bw.dgates)):
        for _ in range(12):
            i = tuple(int(rng.integers(0, s)) for s in arr.shape)
            args = dict(q=q, k=k, v=v, gates=g)
            hi, lo = arr.copy(), arr.copy()
            hi[i] += eps
            lo[i] -= eps
            args[name] = hi
            lp = loss(args["q"], args["k"], args["v"], args["gates"])
            args[name] = lo
            lm = loss(args["q"], args["k"], args["v"], args["gates"])
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[i]) <= 1e-6 * max(1.0, abs(fd)), (name, i, fd, grad[i])


def test_backward_dense_special_case():
    """With every branch dense (m_cmp=1, T>=all blocks, whole-grid window) and gates (a,b,c), the gradients are
    those of (a+b+c) * dense attention -- the textbook softmax-attention backward, written out in numpy."""
    wl = small(seed=4, n=(40,), m=(1, 4, 16), topk=64)
    orc = oracle_for(wl)
    q, k, v, do = (a.astype(np.float64) for a in (wl.q, wl.k, wl.v, wl.dout))
    g = np.zeros((wl.n_tokens, 4, 3))
    g[..., 0], g[..., 1], g[..., 2] = 0.2, 0.5, 0.8
    f = orc.forward(q, k, v, g)
    bw = orc.backward(q, k, v, g, do, f.topk_idx)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for h in range(4):
        kv = h // 2
        s = (q[:, h] @ k[:, kv].T) * orc.scale
        p = np.exp(s - s.max(1, keepdims=True))
        p /= p.sum(1, keepdims=True)
        go = 1.5 * do[:, h]
        dv[:, kv] += p.T @ go
        dp = go @ v[:, kv].T
        ds = p * (dp - (dp * p).sum(1, keepdims=True)) * orc.scale
        dq[:, h] = ds @ k[:, kv]
        dk[:, kv] += ds.T @ q[:, h]
    np.testing.assert_allclose(bw.dq, dq, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw.dk, dk, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bw.dv, dv, rtol=1e-10, atol=1e-12)
    o, _ = dense_attention(q, k, v, 2, orc.scale)
    np.testing.assert_allclose(bw.dgates, np.repeat((do * o).sum(-1, keepdims=True), 3, -1), rtol=1e-10, atol=1e-12)


# ---- P12: backward is linear in dO; rows with dO = 0 contribute nothing (so a query subsample is exact)
def test_backward_linearity_and_subsampling():
    wl = small(n=(60,))
    orc = oracle_for(wl)
    f = orc.forward(wl.q, wl.k, wl.v, wl.gates)
    sub = np.arange(0, 60, 4, dtype=np.int32)
    masked = np.zeros_like(wl.dout)
    masked[sub] = wl.dout[sub]
    full = orc.backward(wl.q, wl.k, wl.v, wl.gates, masked, f.topk_idx, out_branch=f.out_branch)
    part = orc.backward(wl.q, wl.k, wl.v, wl.gates, wl.dout, f.topk_idx, out_branch=f.out_branch, queries=sub)
    for a, b in ((full.dq, part.dq), (full.dk, part.dk), (full.dv, part.dv), (full.dgates, part.dgates)):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    twice = orc.backward(wl.q, wl.k, wl.v, wl.gates, 2.0 * wl.dout.astype(float), f.topk_idx, out_branch=f.out_branch)
    once = orc.backward(wl.q, wl.k, wl.v, wl.gates, wl.dout, f.topk_idx, out_branch=f.out_branch)
    np.testing.assert_allclose(twice.dk, 2 * once.dk, rtol=1e-12, atol=1e-13)


# ---- P13: block structure: sort, CSR arrays, Morton code
def test_morton_roundtrip_and_order():
    rng = np.random.default_rng(0)
    xyz = rng.integers(0, 128, size=(500, 3))
    code = morton3(xyz[:, 0], xyz[:, 1], xyz[:, 2], 7)
    dec = np.zeros_like(xyz)
    for i in range(7):
        dec[:, 0] |= ((code >> np.uint64(3 * i + 2)) & np.uint64(1)).astype(np.int64) << i
        dec[:, 1] |= ((code >> np.uint64(3 * i + 1)) & np.uint64(1)).astype(np.int64) << i
        dec[:, 2] |= ((code >> np.uint64(3 * i)) & np.uint64(1)).astype(np.int64) << i
    assert np.array_equal(dec, xyz)
    assert int(morton3(np.array([1]), np.array([0]), np.array([0]), 3)[0]) == 4
    assert int(morton3(np.array([0]), np.array([1]), np.array([0]), 3)[0]) == 2
    assert int(morton3(np.array([3]), np.array([0]), np.array([5]), 3)[0]) == 0b001_100_101 | 0  # x=011,z=101


@pytest.mark.parametrize("dup", [False, True])
def test_block_structure_against_python_grouping(dup):
    wl = small(seed=13, grid=16, n=(90, 0, 70), m=(2, 4, 8), dup=dup)
    b = build_blocks(wl.coords, wl.batch_offsets, 16, 2, 4, 8)
    n = wl.n_tokens
    assert sorted(b.perm.tolist()) == list(range(n))
    assert np.array_equal(b.inv_perm[b.perm], np.arange(n))
    item = b.tok_item
    # token order == Python's sorted() on (item, Morton, caller index)
    code = morton3(wl.coords[:, 0], wl.coords[:, 1], wl.coords[:, 2], 4)
    expect = sorted(range(n), key=lambda t: (int(item[t]), int(code[t]), t))
    assert b.perm.tolist() == expect
    for level, m in (("cmp", 2), ("slc", 4), ("win", 8)):
        groups = {}
        for t in range(n):
            groups.setdefault((int(item[t]), *(int(c) // m for c in wl.coords[t])), []).append(t)
        st = b.start[level]
        assert st[0] == 0 and st[-1] == n and np.all(np.diff(st) > 0) and len(st) == len(groups) + 1
        for j in range(len(groups)):
            mem = b.perm[st[j]:st[j + 1]]
            key = (int(item[mem[0]]), *(int(c) // m for c in wl.coords[mem[0]]))
            assert sorted(mem.tolist()) == sorted(groups[key])
            assert np.all(b.ids[level][mem] == j)
    cs = b.slc_child_start
    assert cs[0] == 0 and cs[-1] == b.n_blocks["cmp"] and np.all(np.diff(cs) >= 1) and np.all(np.diff(cs) <= 8)
    for j in range(b.n_blocks["slc"]):
        assert np.all(b.cmp_parent[cs[j]:cs[j + 1]] == j)
    assert b.cmp_batch[1] == b.cmp_batch[2]  # the empty item owns no block
    assert b.cmp_batch[-1] == b.n_blocks["cmp"] and b.slc_batch[-1] == b.n_blocks["slc"]
    assert np.array_equal(b.tok_win, b.ids["win"][b.perm])


def test_block_arrays_stay_in_bounds():
    """The bounds rule the GPU tests apply to the arrays a handle exports, applied to the oracle's own arrays (voxel
    grids with duplicates and empty items, and sequences): a rule the reference itself broke would prove nothing."""
    from oracle.blocks import build_blocks_1d
    from oracle.compare import check_block_arrays
    cases = [inputs.random_points_workload(5, 16, (90, 0, 70), 2, 1, 8, (2, 4, 8), 2),
             inputs.random_points_workload(6, 4, (200,), 2, 1, 8, (1, 2, 4), 2, allow_duplicates=True),
             inputs.make_workload("tiny", with_tensors=False)]
    for wl in cases:
        b = build_blocks(wl.coords, wl.batch_offsets, wl.grid, wl.m_cmp, wl.m_slc, wl.m_win)
        arr = dict(perm=b.perm, inv_perm=b.inv_perm, cmp_start=b.start["cmp"], slc_start=b.start["slc"], win_start=b.start["win"],
                   slc_child_start=b.slc_child_start, cmp_batch=b.cmp_batch, slc_batch=b.slc_batch, tok_win=b.tok_win)
        check_block_arrays(arr, wl.n_tokens, wl.n_batch)
    offs = np.array([0, 70, 70, 333], dtype=np.int32)
    b = build_blocks_1d(offs, 6, 18, 25)
    arr = dict(perm=b.perm, inv_perm=b.inv_perm, cmp_start=b.start["cmp"], slc_start=b.start["slc"], win_start=b.start["win"],
               slc_child_start=b.slc_child_start, cmp_batch=b.cmp_batch, slc_batch=b.slc_batch, tok_win=b.tok_win)
    check_block_arrays(arr, 333, 3)
    bad = dict(arr)
    bad["slc_start"] = arr["slc_start"].copy()
    bad["slc_start"][1] = bad["slc_start"][2]          # a planted empty block must be caught
    with pytest.raises(AssertionError):
        check_block_arrays(bad, 333, 3)
