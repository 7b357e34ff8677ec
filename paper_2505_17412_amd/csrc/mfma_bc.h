// Staging of whole key blocks into LDS and the work-chunk lookup of the block-centric selection kernels (gfx950,
// wave64); the tile layout itself (PTile) is the one of mfma_qc.h.
#pragma once

#include "mfma_qc.h"

// Copy rows r0 .. r0 + 32*ntiles - 1 of two row-major arrays (already offset to the KV group or head group; `stride`
// elements between rows) into LDS tiles of the layout above.
template <int D, bool SWZ, int NTHR>
__device__ inline void p_stage2(const bf16_t *xa, const bf16_t *xb, uint32_t stride, int r0, int ntiles, unsigned char *ta,
                                unsigned char *tb) {
  using P = PTile<D, SWZ>;
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
