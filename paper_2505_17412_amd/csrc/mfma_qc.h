// Query-centric tile pipeline shared by the forward and the dQ kernels (gfx950, wave64).
//
// A workgroup of 4 wavefronts owns 4*CB*16 query rows (consecutive sorted tokens x the heads of one KV group);
// each wavefront keeps CB blocks of 16 query columns in registers.  The workgroup walks a list of key ranges
// (one range for the compression and window branches, the union of the selected blocks for the selection
// branch).  Every 32-key tile is loaded once per workgroup, global -> registers -> LDS, double buffered so the
// loads of tile i+1 fly while tile i is consumed; all four wavefronts then take their MFMA A operands from LDS.
#pragma once

#include "mfma_common.h"

// LDS geometry of one staged tile set.  Row-major tiles: 32 key rows of D (+8 pad) bf16, 16-byte segments XOR
// swizzled by bit 3 of the row so that the rows {0-3, 8-11} (and {4-7, 12-15}, ...) an operand read touches in
// one 8-lane phase fall into different 16-byte bank groups.  Transposed tiles: D rows (dims) of 32 keys (+8 pad).
template <int D>
struct TileGeom {
  static constexpr int KROW = D + 8;
  static constexpr int ROW_ELEMS = 32 * KROW;
  static constexpr int TROW = 40;
  static constexpr int T_ELEMS = D * TROW;
  static constexpr int ROW_ITEMS = 32 * D / 8;                  // 16-byte items of a row-major tile
  static constexpr int T_ITEMS = 4 * D;                         // 16-byte items of a transposed tile
  static constexpr int ROW_PER_THREAD = (ROW_ITEMS + 255) / 256;
  static constexpr int T_PER_THREAD = (T_ITEMS + 255) / 256;
  __device__ static inline int swz(int row) { return D >= 64 ? ((row >> 3) & 1) * 4 : 0; }
  // element offset of (row, 16-byte segment) inside a row-major tile
  __device__ static inline int row_off(int row, int seg) { return row * KROW + ((seg ^ swz(row)) << 3); }
  // element offset of (dim, chunk of 8 keys) inside a transposed tile
  __device__ static inline int t_off(int dim, int chunk) { return dim * TROW + (chunk << 3); }
};

// Registers holding one tile set on its way from global memory to LDS.
template <int D, int NROW, int NT>
struct TileRegs {
  bf16x8 r[NROW][TileGeom<D>::ROW_PER_THREAD];
  bf16x8 t[NT][TileGeom<D>::T_PER_THREAD];
};

// Global sources of a tile set: row-major arrays [rows][Hkv][D] and chunk-transposed arrays [rows/8][Hkv][D][8],
// already offset to the KV group.
template <int NROW, int NT>
struct TileSrc {
  const bf16_t *row[NROW];
  const bf16_t *tr[NT];
  size_t kstride;  // elements between consecutive rows of a row-major array (Hkv*D)
};

template <int D, int NROW, int NT>
__device__ inline void tile_load(TileRegs<D, NROW, NT> &regs, const TileSrc<NROW, NT> &src, int kb) {
  using G = TileGeom<D>;
#pragma unroll
  for (int x = 0; x < NROW; ++x)
#pragma unroll
    for (int i = 0; i < G::ROW_PER_THREAD; ++i) {
      const int it = threadIdx.x + 256 * i;
      if (G::ROW_ITEMS % 256 == 0 || it < G::ROW_ITEMS) {
        const int row = it / (D / 8), seg = it % (D / 8);
        regs.r[x][i] = ld8(src.row[x] + (size_t)(kb + row) * src.kstride + seg * 8);
      }
    }
#pragma unroll
  for (int x = 0; x < NT; ++x)
#pragma unroll
    for (int i = 0; i < G::T_PER_THREAD; ++i) {
      const int it = threadIdx.x + 256 * i;
      if (G::T_ITEMS % 256 == 0 || it < G::T_ITEMS) {
        const int chunk = it / D, dim = it % D;
        regs.t[x][i] = ld8(src.tr[x] + (size_t)((kb >> 3) + chunk) * src.kstride * 8 + (size_t)dim * 8);
      }
    }
}

// LDS buffer layout of one stage: NROW row-major tiles, then NT transposed tiles.
template <int D, int NROW, int NT>
struct StageLayout {
  static constexpr int ELEMS = NROW * TileGeom<D>::ROW_ELEMS + NT * TileGeom<D>::T_ELEMS;
  __device__ static inline bf16_t *row_tile(bf16_t *stage, int x) { return stage + x * TileGeom<D>::ROW_ELEMS; }
  __device__ static inline bf16_t *t_tile(bf16_t *stage, int x) {
    return stage + NROW * TileGeom<D>::ROW_ELEMS + x * TileGeom<D>::T_ELEMS;
  }
};

template <int D, int NROW, int NT>
__device__ inline void tile_store(const TileRegs<D, NROW, NT> &regs, bf16_t *stage) {
  using G = TileGeom<D>;
  using L = StageLayout<D, NROW, NT>;
#pragma unroll
  for (int x = 0; x < NROW; ++x)
#pragma unroll
    for (int i = 0; i < G::ROW_PER_THREAD; ++i) {
      const int it = threadIdx.x + 256 * i;
      if (G::ROW_ITEMS % 256 == 0 || it < G::ROW_ITEMS) {
        const int row = it / (D / 8), seg = it % (D / 8);
        *reinterpret_cast<bf16x8 *>(L::row_tile(stage, x) + G::row_off(row, seg)) = regs.r[x][i];
      }
    }
#pragma unroll
  for (int x = 0; x < NT; ++x)
#pragma unroll
    for (int i = 0; i < G::T_PER_THREAD; ++i) {
      const int it = threadIdx.x + 256 * i;
      if (G::T_ITEMS % 256 == 0 || it < G::T_ITEMS) {
        const int chunk = it / D, dim = it % D;
        *reinterpret_cast<bf16x8 *>(L::t_tile(stage, x) + G::t_off(dim, chunk)) = regs.t[x][i];
      }
    }
}

// A operand of sub-tile a, contraction step ks, from a row-major LDS tile (row = key, see tile_key_row).
template <int D>
__device__ inline bf16x8 lds_row_operand(const bf16_t *tile, int a, int ks) {
  const int n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
  const int row = 8 * (n >> 2) + 4 * a + (n & 3);
  return *reinterpret_cast<const bf16x8 *>(tile + TileGeom<D>::row_off(row, 4 * ks + quad));
}
// A operand of dim block dt from a transposed LDS tile (row = dim 16*dt + n, keys 8*quad .. +7).
template <int D>
__device__ inline bf16x8 lds_t_operand(const bf16_t *tile, int dt) {
  const int n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
  return *reinterpret_cast<const bf16x8 *>(tile + TileGeom<D>::t_off(16 * dt + n, quad));
}

// Cursor over the tiles of a list of key ranges held in LDS (rng_s/rng_e), uniform across the workgroup.
struct TileIter {
  int r, kb;
};
__device__ inline int lds_uniform(const int *p) { return __builtin_amdgcn_readfirstlane(*p); }
__device__ inline TileIter iter_begin(const int *rng_s, int nr) {
  TileIter it{0, 0};
  if (nr > 0) it.kb = lds_uniform(rng_s) & ~7;
  return it;
}
__device__ inline TileIter iter_next(TileIter it, const int *rng_s, const int *rng_e, int nr) {
  it.kb += 32;
  if (it.kb >= lds_uniform(rng_e + it.r)) {
    ++it.r;
    if (it.r < nr) it.kb = lds_uniform(rng_s + it.r) & ~7;
  }
  return it;
}
