"""Seeded synthetic inputs for Spatial Sparse Attention (SSA).

Stand-ins for the latent sparse-voxel tokens of a 3D shape (the paper's tokens come from
an SDF shell encoded by its VAE, Sec. "Sparse SDF VAE" eq. (1); token counts per resolution are
listed in the DiT training-configuration table).  This module holds no SSA arithmetic: it only
draws voxel coordinates on an analytic signed-distance shell and Gaussian Q/K/V/gates/dO, so
both the CPU oracle and the HIP path can be fed the very same arrays.

Everything is deterministic from ``numpy.random.default_rng(seed)``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------------------------
# analytic signed-distance primitives, evaluated on the integer voxel lattice
# --------------------------------------------------------------------------------------------


def _sdf_sphere(p: np.ndarray, c: np.ndarray, r: float) -> np.ndarray:
    return np.linalg.norm(p - c, axis=-1) - r


def _sdf_box(p: np.ndarray, c: np.ndarray, h: np.ndarray) -> np.ndarray:
    q = np.abs(p - c) - h
    outside = np.linalg.norm(np.maximum(q, 0.0), axis=-1)
    inside = np.minimum(np.max(q, axis=-1), 0.0)
    return outside + inside


def _sdf_torus(p: np.ndarray, c: np.ndarray, R: float, r: float) -> np.ndarray:
    q = p - c
    ring = np.linalg.norm(q[..., :2], axis=-1) - R
    return np.sqrt(ring * ring + q[..., 2] ** 2) - r


def shell_coords(
    seed: int,
    grid: int,
    n_prims: int,
    kinds: Sequence[str],
    width: float,
    size_factor: float = 1.0,
    shuffle: bool = True,
) -> np.ndarray:
    """Voxels of a ``grid``^3 lattice whose |SDF| to a union of random primitives is < ``width``.

    Returns int32 ``[N, 3]`` coordinates, shuffled (tokens arrive in no spatial order).
    Base sizes are given for a 32^3 grid and scale with ``grid / 32``; ``size_factor`` scales the
    primitive sizes (not the centres).
    """
    rng = np.random.default_rng(seed)
    sc = grid / 32.0
    ax = np.arange(grid, dtype=np.float64)
    p = np.stack(np.meshgrid(ax, ax, ax, indexing="ij"), axis=-1)  # [G,G,G,3]
    sdf = np.full((grid, grid, grid), np.inf)
    for _ in range(n_prims):
        kind = kinds[int(rng.integers(0, len(kinds)))]
        c = rng.uniform(8.0, 24.0, size=3) * sc
        if kind == "sphere":
            r = rng.uniform(4.0, 9.0) * sc * size_factor
            d = _sdf_sphere(p, c, r)
        elif kind == "box":
            h = rng.uniform(3.0, 8.0, size=3) * sc * size_factor
            d = _sdf_box(p, c, h)
        elif kind == "torus":
            R = rng.uniform(4.0, 8.0) * sc * size_factor
            r = rng.uniform(1.0, 2.5) * sc * size_factor
            d = _sdf_torus(p, c, R, r)
        else:
            raise ValueError(f"unknown primitive kind {kind!r}")
        sdf = np.minimum(sdf, d)
    coords = np.argwhere(np.abs(sdf) < width).astype(np.int32)  # row-major order
    if shuffle:
        coords = coords[rng.permutation(coords.shape[0])]
    return np.ascontiguousarray(coords)


# --------------------------------------------------------------------------------------------
# bf16 rounding of inputs (round-to-nearest-even), so both sides see identical values
# --------------------------------------------------------------------------------------------


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of ``round_to_bf16(x)``."""
    r = round_to_bf16(x)
    return (r.view(np.uint32) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


# --------------------------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------------------------


@dataclass
class Workload:
    """One synthetic SSA problem instance."""

    name: str
    grid: int
    coords: np.ndarray  # int32 [N,3], caller (shuffled) order
    batch_offsets: np.ndarray  # int32 [B+1]
    n_heads_q: int
    n_heads_kv: int
    head_dim: int
    m_cmp: int
    m_slc: int
    m_win: int
    topk: int
    dtype: str  # "bf16" | "f32"
    q: np.ndarray = field(repr=False, default=None)  # float32 [N,Hq,d] (bf16-representable if dtype=="bf16")
    k: np.ndarray = field(repr=False, default=None)  # float32 [N,Hkv,d]
    v: np.ndarray = field(repr=False, default=None)
    gates: np.ndarray = field(repr=False, default=None)  # float32 [N,Hq,3], order (cmp, slc, win)
    dout: np.ndarray = field(repr=False, default=None)  # float32 [N,Hq,d]
    seeds: Tuple[int, ...] = ()
    dims: int = 3  # 3: voxel grid; 1: sequences (coords then hold (0,0,position) and m_* are block lengths in tokens)

    @property
    def n_tokens(self) -> int:
        return int(self.coords.shape[0])

    @property
    def n_batch(self) -> int:
        return int(self.batch_offsets.shape[0] - 1)


def draw_tensors(
    seed: int, n: int, hq: int, hkv: int, d: int, dtype: str
) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Q,K,V ~ N(0,1); gates = sigmoid(N(0,1)); dO ~ N(0,1); rounded to bf16 when asked."""
    rng = np.random.default_rng(seed + 7919)
    q = rng.standard_normal((n, hq, d), dtype=np.float32)
    k = rng.standard_normal((n, hkv, d), dtype=np.float32)
    v = rng.standard_normal((n, hkv, d), dtype=np.float32)
    z = rng.standard_normal((n, hq, 3), dtype=np.float32)
    gates = (1.0 / (1.0 + np.exp(-z))).astype(np.float32)
    dout = rng.standard_normal((n, hq, d), dtype=np.float32)
    if dtype == "bf16":
        q, k, v, gates, dout = (round_to_bf16(a) for a in (q, k, v, gates, dout))
    return q, k, v, gates, dout


# name -> recipe.  ``kinds`` are the allowed primitive kinds; ``f`` the size factor; ``w`` the
# shell half-width.  H_kv = 2 for the 16-head configs follows the paper's "2 groups" GQA setting
# (Implementation Details, DiT paragraph); the 4-head tiny config uses H_kv = 2 as well.
CONFIGS: Dict[str, dict] = {
    "tiny": dict(seed=1001, grid=32, n_prims=3, kinds=("sphere",), f=1.0, w=1.0,
                 hq=4, hkv=2, d=32, m=(4, 8, 8), topk=4, dtype="f32"),
    "g64": dict(seed=1002, grid=64, n_prims=6, kinds=("sphere", "box"), f=1.0, w=1.0,
                hq=16, hkv=2, d=64, m=(4, 8, 8), topk=8, dtype="bf16"),
    "g128": dict(seed=1003, grid=128, n_prims=10, kinds=("sphere", "box", "torus"), f=0.55, w=1.5,
                 hq=16, hkv=2, d=64, m=(4, 8, 8), topk=16, dtype="bf16"),
    "g128_thick": dict(seed=1008, grid=128, n_prims=10, kinds=("sphere", "box", "torus"), f=0.65, w=3.0,
                       hq=16, hkv=2, d=128, m=(4, 8, 8), topk=16, dtype="bf16"),
}


def make_workload(name: str, with_tensors: bool = True, **overrides) -> Workload:
    """Build one of the named single-shape workloads (``CONFIGS``), optionally overriding fields."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    coords = shell_coords(cfg["seed"], cfg["grid"], cfg["n_prims"], cfg["kinds"], cfg["w"], cfg["f"])
    n = coords.shape[0]
    wl = Workload(
        name=name, grid=cfg["grid"], coords=coords,
        batch_offsets=np.array([0, n], dtype=np.int32),
        n_heads_q=cfg["hq"], n_heads_kv=cfg["hkv"], head_dim=cfg["d"],
        m_cmp=cfg["m"][0], m_slc=cfg["m"][1], m_win=cfg["m"][2], topk=cfg["topk"],
        dtype=cfg["dtype"], seeds=(cfg["seed"],),
    )
    if with_tensors:
        wl.q, wl.k, wl.v, wl.gates, wl.dout = draw_tensors(cfg["seed"], n, cfg["hq"], cfg["hkv"], cfg["d"], cfg["dtype"])
    return wl


def make_batch_workload(
    seeds: Sequence[int] = (1004, 1005, 1006, 1007),
    grid: int = 128,
    n_range: Tuple[int, int] = (20000, 70000),
    hq: int = 16, hkv: int = 2, d: int = 64,
    m: Tuple[int, int, int] = (4, 8, 8), topk: int = 16, dtype: str = "bf16",
    with_tensors: bool = True,
) -> Workload:
    """Variable-length batch: independent shapes concatenated, with int32 batch offsets.

    Per item the size factor is U[0.4,0.5] and the shell half-width U[0.8,1.8]; an item whose token
    count misses ``n_range`` is redrawn with seed += 100.
    """
    items: List[np.ndarray] = []
    used: List[int] = []
    for s in seeds:
        seed = s
        while True:
            rng = np.random.default_rng(seed + 31)
            f = float(rng.uniform(0.4, 0.5))
            w = float(rng.uniform(0.8, 1.8))
            c = shell_coords(seed, grid, 10, ("sphere", "box", "torus"), w, f)
            if n_range[0] <= c.shape[0] <= n_range[1]:
                break
            seed += 100
        items.append(c)
        used.append(seed)
    coords = np.ascontiguousarray(np.concatenate(items, axis=0))
    offs = np.zeros(len(items) + 1, dtype=np.int32)
    offs[1:] = np.cumsum([c.shape[0] for c in items])
    n = coords.shape[0]
    wl = Workload(
        name="batch4", grid=grid, coords=coords, batch_offsets=offs,
        n_heads_q=hq, n_heads_kv=hkv, head_dim=d, m_cmp=m[0], m_slc=m[1], m_win=m[2],
        topk=topk, dtype=dtype, seeds=tuple(used),
    )
    if with_tensors:
        wl.q, wl.k, wl.v, wl.gates, wl.dout = draw_tensors(used[0], n, hq, hkv, d, dtype)
    return wl


def random_points_workload(
    seed: int, grid: int, n_per_item: Sequence[int], hq: int, hkv: int, d: int,
    m: Tuple[int, int, int], topk: int, dtype: str = "f32", allow_duplicates: bool = False,
) -> Workload:
    """Small unstructured test problem: uniformly random voxels per batch item."""
    rng = np.random.default_rng(seed)
    items = []
    for n_i in n_per_item:
        if allow_duplicates:
            c = rng.integers(0, grid, size=(n_i, 3), dtype=np.int64)
        else:
            flat = rng.choice(grid ** 3, size=n_i, replace=False)
            c = np.stack(np.unravel_index(flat, (grid, grid, grid)), axis=-1)
        items.append(c.astype(np.int32))
    coords = np.ascontiguousarray(np.concatenate(items, axis=0)) if items else np.zeros((0, 3), np.int32)
    offs = np.zeros(len(items) + 1, dtype=np.int32)
    offs[1:] = np.cumsum([c.shape[0] for c in items])
    n = coords.shape[0]
    wl = Workload(
        name=f"rand{seed}", grid=grid, coords=coords, batch_offsets=offs,
        n_heads_q=hq, n_heads_kv=hkv, head_dim=d, m_cmp=m[0], m_slc=m[1], m_win=m[2],
        topk=topk, dtype=dtype, seeds=(seed,),
    )
    wl.q, wl.k, wl.v, wl.gates, wl.dout = draw_tensors(seed, n, hq, hkv, d, dtype)
    return wl


def make_sequence_workload(
    seed: int, lens: Sequence[int], hq: int = 16, hkv: int = 2, d: int = 64,
    l: Tuple[int, int, int] = (32, 64, 512), topk: int = 16, dtype: str = "bf16", with_tensors: bool = True,
) -> Workload:
    """Sequences of the given lengths with a one-dimensional partition: compression blocks of l[0] tokens, selection
    blocks of l[1], windows of l[2] (the block sizes of the sequence models whose partition the paper replaces)."""
    offs = np.concatenate([[0], np.cumsum(np.asarray(lens, dtype=np.int64))]).astype(np.int32)
    n = int(offs[-1])
    coords = np.zeros((n, 3), dtype=np.int32)
    for i in range(len(lens)):
        coords[offs[i]:offs[i + 1], 2] = np.arange(int(lens[i]), dtype=np.int32)
    wl = Workload(
        name="seq1d", grid=0, coords=coords, batch_offsets=offs, n_heads_q=hq, n_heads_kv=hkv, head_dim=d,
        m_cmp=l[0], m_slc=l[1], m_win=l[2], topk=topk, dtype=dtype, seeds=(seed,), dims=1,
    )
    if with_tensors:
        wl.q, wl.k, wl.v, wl.gates, wl.dout = draw_tensors(seed, n, hq, hkv, d, dtype)
    return wl
