// Shared pieces of the bf16 MFMA kernels (gfx950, wave64, v_mfma_f32_16x16x32_bf16).
//
// Operand convention used throughout (hardware layout of the 16x16x32 instruction):
//   A (16 x 32): lane l supplies row (l & 15), contraction indices 8*(l >> 4) .. +7   (8 bf16 = 16 bytes)
//   B (32 x 16): lane l supplies column (l & 15), contraction indices 8*(l >> 4) .. +7
//   C/D (16 x 16 fp32): lane l holds column (l & 15), rows 4*(l >> 4) .. +3
// "quad" below is l >> 4, "n" is l & 15.
//
// Key-tile convention: a tile covers 32 consecutive rows kb..kb+31 of a key array, kb a multiple of 8.  It is
// processed as two 16-row sub-tiles whose row r maps to key kb + 8*(r >> 2) + 4*a + (r & 3) (a = sub-tile), so
// that after the two MFMAs lane l holds the eight CONSECUTIVE keys kb + 8*quad .. +7 of column n -- exactly
// the contraction slice the next MFMA wants from it as a B operand, with no cross-lane movement.
#pragma once

#include "ssa_internal.h"

typedef uint16_t bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__device__ inline bf16x8 ld8(const bf16_t *p) { return *reinterpret_cast<const bf16x8 *>(p); }
__device__ inline bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.0f;
  return z;
}
__device__ inline f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// All-ones A operand of the matrix instruction (sums the 32 contraction entries of every column).  Build it once per
// kernel: the empty asm makes the value opaque, so it stays in its four registers instead of being rebuilt with
// three moves in front of every use.
__device__ inline bf16x8 ones_operand() {
  const float w1 = __builtin_bit_cast(float, 0x3F803F80u);  // two bf16 ones
  f32x4 w = {w1, w1, w1, w1};
  asm volatile("" : "+v"(w));
  return __builtin_bit_cast(bf16x8, w);
}
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ inline int wave_min_i(int v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = min(v, __shfl_xor(v, off));
  return v;
}
__device__ inline int wave_max_i(int v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = max(v, __shfl_xor(v, off));
  return v;
}

// Sum over aligned groups of hs lanes (hs a power of two <= 16) inside each 16-lane row, with DPP lane
// permutations only (no LDS traffic): xor 1, xor 2 by quad permutes; once the lanes of a quad agree, the
// half-row and row mirrors act as xor 4 and xor 8.
template <int CTRL>
__device__ inline float dpp_add(float v) {
  return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
__device__ inline float group_sum(float v, int hs) {
  if (hs >= 2) v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
  if (hs >= 4) v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
  if (hs >= 8) v = dpp_add<0x141>(v);   // row_half_mirror
  if (hs >= 16) v = dpp_add<0x140>(v);  // row_mirror
  return v;
}

// Dims of an accumulator whose rows came from a transposed tile operand.  The transposing LDS read takes the 16 rows
// of dim block dt from two 16-byte segments of a row that lie 32 bytes apart (see PTile in mfma_qc.h: that pairing is
// what keeps the read free of bank conflicts), so the block covers dims b .. b + 7 and b + 16 .. b + 23 with
// b = 32*(dt >> 1) + 8*(dt & 1).  tr_dim: dim of row n of the block; acc_dim: the first of the 4 consecutive dims that a
// lane of row group `quad` holds in its accumulator register of block dt (C layout: rows 4*quad .. +3).
__device__ inline int tr_dim(int dt, int n) { return 32 * (dt >> 1) + 8 * (dt & 1) + 16 * (n >> 3) + (n & 7); }
__device__ inline int acc_dim(int dt, int quad) { return tr_dim(dt, 4 * quad); }

// Store the accumulator tile of one query column block to row-major rows of D bf16: on entry lane (n, quad) holds, for
// every dim block dt, the 4 dims acc_dim(dt, quad) .. +3 of column n, i.e. 8 bytes in each of D/16 places of its row.
// Within a group of four dim blocks (64 dims) the dim index is 32*dt1 + 16*quad1 + 8*dt0 + 4*quad0 + i (dt1, dt0 and
// quad1, quad0 the bits of dt & 3 and of quad): exchanging dt1 with quad0 (one round of v_permlane16_swap: lanes 16
// apart hold the same column) leaves every lane with 16 consecutive dims, so a row goes out as 32-byte pieces, four
// lanes covering 64 consecutive dims, instead of 8-byte pieces.  `row`: this lane's row (column n); scale: factor
// applied before rounding; lanes with !valid take part in the exchange and store nothing.  D = 64 or 128.
template <int D>
__device__ inline void store_row_tile_if(bf16_t *row, const f32x4 (&o)[D / 16], float scale, bool valid) {
  static_assert(D % 64 == 0, "groups of four dim blocks");
  const int quad = threadIdx.x >> 4 & 3;
#pragma unroll
  for (int h = 0; h < D / 64; ++h) {
    unsigned lo[4], hi[4];  // packed bf16 pairs: dims (0,1) and (2,3) of the lane's 4-dim group of dim block 4*h + j
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x4 x;
#pragma unroll
      for (int i = 0; i < 4; ++i) x[i] = (__bf16)(o[4 * h + j][i] * scale);
      typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
      const u32x2 w = __builtin_bit_cast(u32x2, x);
      lo[j] = w[0];
      hi[j] = w[1];
    }
    auto swap16 = [](unsigned &a, unsigned &b) {  // odd 16-lane rows of a <-> even 16-lane rows of b
      const auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
      a = r[0]; b = r[1];
    };
    swap16(lo[0], lo[2]); swap16(hi[0], hi[2]); swap16(lo[1], lo[3]); swap16(hi[1], hi[3]);
    // register j = 2*j1 + j0 now holds dims 64*h + 32*quad0 + 16*quad1 + 8*j0 + 4*j1 .. +3
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    if (valid) {
      u32x4 *dst = reinterpret_cast<u32x4 *>(row + 64 * h + 32 * (quad & 1) + 16 * (quad >> 1));
      // written once, read once much later by the merge kernel: streaming stores, so the rows do not push the query
      // rows (which every selected block reads again) out of the caches
      __builtin_nontemporal_store(u32x4{lo[0], hi[0], lo[2], hi[2]}, dst);
      __builtin_nontemporal_store(u32x4{lo[1], hi[1], lo[3], hi[3]}, dst + 1);
    }
  }
}

// One row of D bf16 per query column from the accumulator tile `o` (unscaled); lanes with !valid store nothing (the
// lanes of a column agree on valid).  Wide stores where the dim blocks come in fours, 8-byte pieces otherwise.
template <int D>
__device__ inline void store_partial_row(bf16_t *row, const f32x4 (&o)[D / 16], bool valid) {
  if constexpr (D % 64 == 0) {
    store_row_tile_if<D>(row, o, 1.0f, valid);  // the lane exchange runs with every lane on; only the stores are conditional
  } else {
    const int quad = threadIdx.x >> 4 & 3;
    if (valid) {
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        bf16x4 x;
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = (__bf16)o[dt][i];
        *reinterpret_cast<bf16x4 *>(row + acc_dim(dt, quad)) = x;
      }
    }
  }
}

// Row of the A operand a lane feeds for sub-tile `a` of the key tile starting at kb.
__device__ inline int tile_key_row(int kb, int a) {
  const int r = threadIdx.x & 15;
  return kb + 8 * (r >> 2) + 4 * a + (r & 3);
}

// Device arrays of the block structure and the sorted K,V copies the kernels read.
struct MfmaView {
  const int32_t *perm, *tok_item, *tok_win, *cmp_start, *slc_start, *win_start, *cmp_slc, *cmp_batch, *slc_batch,
      *item_start;
  int N, Nc, Ns, Hq, Hkv, hs, T, s_max;
  float scale, sl2;  // softmax scale, scale * log2(e)
  // sorted copies (bf16), row-major [rows][Hkv][D]: token K, V and pooled K, V
  const bf16_t *Ks, *Vs, *Kc, *Vc;
};
