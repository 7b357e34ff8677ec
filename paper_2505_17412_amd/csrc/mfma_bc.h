// LDS tile layout and work-chunk lookup of the block-centric selection kernels (gfx950, wave64).
//
// A 32-row tile of a row-major bf16 array is kept as D/8 planes, one per 16-byte segment of a row; a plane holds the
// 32 rows' segments in the slot order sigma(row) (the order in which the lanes of the two 16-row matrix sub-tiles read
// them, see TileGeom) and is followed by 64 bytes of padding.  Every operand address is then lane part + compile-time
// constant: the sub-tile, the contraction step, the output-dim block and the tile index all move the address by
// constants, which the LDS instructions take as immediate offsets, so a tile costs no address arithmetic at all.  The
// padding shifts consecutive planes by 16 banks: the 16 lanes of a transposing read (two planes, four rows each) and
// the 64 lanes of a staging write (eight planes) spread evenly over the banks.
#pragma once

#include "mfma_qc.h"

template <int D>
struct PTile {
  static constexpr int SEGS = D / 8;
  static constexpr int PLANE_B = 32 * 16 + 64;   // bytes per plane
  static constexpr int BYTES = SEGS * PLANE_B;   // bytes per 32-row tile
  static constexpr int ITEMS = 32 * SEGS;        // 16-byte items per tile
  __device__ static inline int off(int row, int seg) { return seg * PLANE_B + TileGeom<D>::sigma(row) * 16; }
  // lane part of the address of a row operand (A or B operand whose rows are the tile's rows): sub-tile a and
  // contraction step ks add a*256 + ks*4*PLANE_B
  __device__ static inline int row_lane() { return (int)(threadIdx.x >> 4 & 3) * PLANE_B + (int)(threadIdx.x & 15) * 16; }
  // lane part of the address of a transposed operand (rows = dims 16*dt + n, contraction over the tile's rows
  // 8*quad .. +7): dim block dt adds dt*2*PLANE_B, the second half (rows +4 .. +7) adds 256
  __device__ static inline int tr_lane() {
    const int p = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
    return ((p & 3) >> 1) * PLANE_B + (4 * quad + (p >> 2)) * 16 + (p & 1) * 8;
  }
};

typedef const __attribute__((address_space(3))) unsigned char *lds_cptr;

template <int D>
__device__ inline bf16x8 p_row_operand(lds_cptr lane_base, int a, int ks) {
  return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8 *>(lane_base + a * 256 + ks * 4 * PTile<D>::PLANE_B);
}

template <int D>
__device__ inline bf16x8 p_tr_operand(lds_cptr lane_base, int dt) {
  typedef __attribute__((address_space(3))) s16x4 *tr_ptr;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(lane_base + dt * 2 * PTile<D>::PLANE_B));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(lane_base + dt * 2 * PTile<D>::PLANE_B + 256));
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

// Copy rows r0 .. r0 + 32*ntiles - 1 of two row-major arrays (already offset to the KV group or head group; `stride`
// elements between rows) into LDS tiles of the layout above.
template <int D, int NTHR>
__device__ inline void p_stage2(const bf16_t *xa, const bf16_t *xb, uint32_t stride, int r0, int ntiles, unsigned char *ta,
                                unsigned char *tb) {
  using P = PTile<D>;
  const int total = ntiles * P::ITEMS;
  for (int i0 = 0; i0 < total; i0 += 4 * NTHR) {
    bf16x8 ra[4], rb[4];
    int off[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int it = i0 + u * NTHR + (int)threadIdx.x;
      off[u] = -1;
      if (it < total) {
        const int t = it / P::ITEMS, w = it % P::ITEMS, row = w / P::SEGS, seg = w % P::SEGS;
        const uint32_t src = (uint32_t)(r0 + 32 * t + row) * stride + (uint32_t)(seg * 8);
        ra[u] = ld8(xa + src);
        rb[u] = ld8(xb + src);
        off[u] = t * P::BYTES + P::off(row, seg);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (off[u] >= 0) {
        *reinterpret_cast<bf16x8 *>(ta + off[u]) = ra[u];
        *reinterpret_cast<bf16x8 *>(tb + off[u]) = rb[u];
      }
  }
}

// Work chunk -> (key, chunk inside the key) by bisection over the chunk prefix sums; false when w is past the end.
__device__ inline bool bc_find_chunk(const int32_t *chunk_start, int nkeys, int w, int &key, int &chunk) {
  if (w >= chunk_start[nkeys]) return false;
  int lo = 0, hi = nkeys;  // chunk_start[lo] <= w < chunk_start[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (chunk_start[mid] <= w) lo = mid; else hi = mid;
  }
  key = lo;
  chunk = w - chunk_start[lo];
  return true;
}

// Workgroup id -> work chunk.  Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2); the map
// gives every XCD one contiguous run of the `total` chunks (one KV head, neighbouring blocks), so a block's rows are
// fetched into one L2.  The grid is a multiple of 8 workgroups; ids past the end return -1.
__device__ inline int bc_chunk_of_workgroup(int total) {
  const int per = (total + 7) >> 3, xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
  const int w = xcd * per + i;
  return (i < per && w < total) ? w : -1;
}
