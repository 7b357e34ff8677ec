// LDS tile layout of all attention kernels, and the query-centric tile pipeline of the compression and window
// kernels, forward and dQ (gfx950, wave64).
//
// Pipeline: a workgroup of 4 wavefronts owns 4*CB*16 query rows (consecutive sorted tokens x the heads of one KV
// group); each wavefront keeps CB blocks of 16 query columns in registers.  The workgroup walks a contiguous key range
// (the item's pooled keys, the token's window).  Every 32-key tile is loaded once per workgroup, global -> registers ->
// LDS, double buffered so the loads of the next tiles fly while a tile is consumed; all four wavefronts then take their
// MFMA A operands from LDS.  (The selection branch has kernels of its own: see mfma_bc.h.)
#pragma once

#include "mfma_common.h"
#include "topk_device.h"

// LDS geometry of one staged tile set.
// Row-major tiles (32 rows of D bf16, no padding) are stored as [16-byte segment][row slot][8 elements]: the slot of
// row k is sigma(k) = 16*((k>>2)&1) + 4*(k>>3) + (k&3), i.e. the 16 rows lane n = 0..15 of sub-tile a reads (see
// tile_key_row) occupy the consecutive slots 16a .. 16a+15, so one operand read of a 16-lane quad covers 256
// contiguous bytes.  The slot is XORed with (segment & 7): reads stay a permutation of the same 16 slots, and the
// 8 threads that stage one row (8 segments, 512 bytes apart) land in 8 different 16-byte bank groups.
template <int D>
struct TileGeom {
  static constexpr int ROW_ELEMS = 32 * D;
  static constexpr int ROW_ITEMS = 32 * D / 8;                  // 16-byte items of a row-major tile
  // 16-byte items per thread when NTHR threads stage a tile
  static constexpr int row_per_thread(int nthr) { return (ROW_ITEMS + nthr - 1) / nthr; }
  __device__ static inline int sigma(int row) { return 16 * ((row >> 2) & 1) + 4 * (row >> 3) + (row & 3); }
  // element offset of (row slot, 16-byte segment) inside a row-major tile
  __device__ static inline int slot_off(int slot, int seg) { return ((seg << 5) + (slot ^ (seg & 7))) << 3; }
  // element offset of (row, 16-byte segment)
  __device__ static inline int row_off(int row, int seg) { return slot_off(sigma(row), seg); }
};

typedef __attribute__((ext_vector_type(4))) short s16x4;

// Tile layout of the attention kernels in LDS.  A 32-row tile of a row-major bf16 array is kept as D/8 planes of 512
// bytes, one per 16-byte segment of a row; a plane holds the 32 rows' segments in the slot order sigma(row) (the order
// in which the lanes of the two 16-row matrix sub-tiles read them).  The slot is XORed with a per-plane constant,
// swz(seg), chosen so that all three access patterns are free of LDS bank conflicts (measured with the LDS counters:
// 0 conflict cycles per instruction for each):
//   * staging writes: the 8 threads that stage one row write 8 planes, 512 bytes apart; the low three bits of swz
//     (seg & 7, present with SWZ only) put them in 8 different 16-byte bank groups.  Kernels that stage a block once
//     and read it many times leave them out (SWZ = false): their lane offsets then differ between contraction steps
//     and between dim blocks by constants only, which saves the registers that hold them;
//   * row operands (16-byte reads): the four quads of a wavefront read planes 4*ks .. 4*ks + 3, each 16 consecutive
//     slots; the two quads served together (0,1 and 2,3) must not differ in bit 3 of swz, so that bit is the same for
//     segments 4*ks, 4*ks + 1 and for 4*ks + 2, 4*ks + 3;
//   * transposed operands (8-byte transposing reads): one read takes 4-element pieces from TWO planes; planes whose
//     swz agrees in bit 3 would collide (they are a multiple of 512 bytes apart), so a dim block pairs segment s with
//     segment s + 2, whose bit 3 differs.  The 16 output rows of dim block dt are therefore not the dims 16*dt .. +15
//     but tr_dim(dt, 0..15): dims 8*s .. 8*s + 7 and 8*s + 16 .. 8*s + 23 with s = tr_seg(dt).  Every consumer of an
//     accumulator indexed by dt goes through acc_dim() (mfma_common.h), which states the same map per lane.
// Operand addresses are lane part + compile-time constant: the lane part depends on the contraction step (row
// operands) or the output-dim block (transposed operands) only through the swizzle, so a kernel keeps D/32 + D/16
// lane offsets in registers (Lanes) and the sub-tile, the row half, the tile index and the LDS stage all move the
// address by constants, which the LDS instructions take as immediate offsets: a tile costs no address arithmetic.
template <int D, bool SWZ = true>
struct PTile {
  static constexpr int SEGS = D / 8;
  static constexpr int PLANE_B = 512;            // bytes per plane: 32 row slots of 16 bytes
  static constexpr int BYTES = SEGS * PLANE_B;   // bytes per 32-row tile
  static constexpr int ITEMS = 32 * SEGS;        // 16-byte items per tile
  __device__ static inline int swz(int seg) { return (SWZ ? seg & 7 : 0) ^ (((seg >> 1) & 1) << 3); }
  __device__ static inline int slot_off(int slot, int seg) { return seg * PLANE_B + ((slot ^ swz(seg)) << 4); }
  __device__ static inline int off(int row, int seg) { return slot_off(TileGeom<D>::sigma(row), seg); }
  // first of the two segments (s, s + 2) that dim block dt of a transposed operand is read from
  __device__ static inline int tr_seg(int dt) { return 4 * (dt >> 1) + (dt & 1); }
  struct Lanes {
    int row[D / 32];  // row operand (rows = the tile's rows), contraction step ks; sub-tile a adds a*256
    int tr[D / 16];   // transposed operand (rows = dims tr_dim(dt, n), contraction over rows 8*quad .. +7); rows +4 .. +7 add 256
  };
  __device__ static inline Lanes lanes() {
    const int n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
    Lanes l;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) l.row[ks] = slot_off(n, 4 * ks + quad);
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) l.tr[dt] = slot_off(4 * quad + (n >> 2), tr_seg(dt) + ((n & 3) >> 1) * 2) + (n & 1) * 8;
    return l;
  }
};

typedef const __attribute__((address_space(3))) unsigned char *lds_cptr;

// A operand of sub-tile a, contraction step ks (row = key, see tile_key_row) from the tile at `tile` (uniform address).
template <int D, bool SWZ = true>
__device__ inline bf16x8 p_row_operand(lds_cptr tile, const typename PTile<D, SWZ>::Lanes &l, int a, int ks) {
  return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8 *>(tile + l.row[ks] + a * 256);
}

// Transposed A operand (row n = dim tr_dim(dt, n), contraction over the tile's rows 8*quad .. +7), taken from the same
// row-major tile with the transposing LDS read of gfx950 (ds_read_b64_tr_b16): inside a 16-lane group lane p hands in
// the address of 4 consecutive elements and lane i receives element (i & 3) of lanes (i >> 2), 4 + (i >> 2),
// 8 + (i >> 2), 12 + (i >> 2).  With lane p pointing at row 8*quad + (p >> 2) and at the 4-dim piece (p & 3) of the
// block (pieces 0, 1 in segment tr_seg(dt), pieces 2, 3 in the segment two further), lane i ends up with dim
// tr_dim(dt, i) of rows 8*quad .. +3; a second read covers rows +4 .. +7.
template <int D, bool SWZ = true>
__device__ inline bf16x8 p_tr_operand(lds_cptr tile, const typename PTile<D, SWZ>::Lanes &l, int dt) {
  typedef __attribute__((address_space(3))) s16x4 *tr_ptr;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(tile + l.tr[dt]));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(tile + l.tr[dt] + 256));
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

// Registers holding one tile set on its way from global memory to LDS.
template <int D, int NROW, int NTHR = 256>
struct TileRegs {
  bf16x8 r[NROW][TileGeom<D>::row_per_thread(NTHR)];
};

// Global sources of a tile set: row-major arrays [rows][Hkv][D], already offset to the KV group.
template <int NROW>
struct TileSrc {
  const bf16_t *row[NROW];
  uint32_t kstride;  // elements between consecutive rows of a row-major array (Hkv*D); whole arrays stay below 2^31 elements
};

template <int D, int NROW, int NTHR>
__device__ inline void tile_load(TileRegs<D, NROW, NTHR> &regs, const TileSrc<NROW> &src, int kb) {
  using G = TileGeom<D>;
#pragma unroll
  for (int x = 0; x < NROW; ++x)
#pragma unroll
    for (int i = 0; i < G::row_per_thread(NTHR); ++i) {
      const int it = threadIdx.x + NTHR * i;
      if (G::ROW_ITEMS % NTHR == 0 || it < G::ROW_ITEMS) {
        const int row = it / (D / 8), seg = it % (D / 8);
        regs.r[x][i] = ld8(src.row[x] + ((uint32_t)(kb + row) * (uint32_t)src.kstride + (uint32_t)(seg * 8)));
      }
    }
}

// LDS buffer layout of one stage: NROW tiles in the padded layout.
template <int D, int NROW>
struct StageLayout {
  static constexpr int TILE_ELEMS = PTile<D>::BYTES / 2;
  static constexpr int ELEMS = NROW * TILE_ELEMS;
  __device__ static inline bf16_t *row_tile(bf16_t *stage, int x) { return stage + x * TILE_ELEMS; }
};

template <int D, int NROW, int NTHR>
__device__ inline void tile_store(const TileRegs<D, NROW, NTHR> &regs, bf16_t *stage) {
  using G = TileGeom<D>;
  using L = StageLayout<D, NROW>;
#pragma unroll
  for (int x = 0; x < NROW; ++x)
#pragma unroll
    for (int i = 0; i < G::row_per_thread(NTHR); ++i) {
      const int it = threadIdx.x + NTHR * i;
      if (G::ROW_ITEMS % NTHR == 0 || it < G::ROW_ITEMS) {
        const int row = it / (D / 8), seg = it % (D / 8);
        *reinterpret_cast<bf16x8 *>((unsigned char *)L::row_tile(stage, x) + PTile<D>::off(row, seg)) = regs.r[x][i];
      }
    }
}

// A operand of sub-tile a, contraction step ks, from a row-major LDS tile (row = key, see tile_key_row).
template <int D>
__device__ inline bf16x8 lds_row_operand(const bf16_t *tile, int a, int ks) {
  const int n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
  return *reinterpret_cast<const bf16x8 *>(tile + TileGeom<D>::slot_off(16 * a + n, 4 * ks + quad));
}

// Transposed A operand (row = dim 16*dt + n, contraction over the tile's rows 8*quad .. +7), taken from the same
// ROW-major LDS tile with the transposing LDS read of gfx950 (ds_read_b64_tr_b16): inside a 16-lane group lane p
// hands in the address of 4 consecutive elements and lane i receives element (i & 3) of lanes (i >> 2), 4 + (i >> 2),
// 8 + (i >> 2), 12 + (i >> 2).  With lane p pointing at row 8*quad + (p >> 2), dims 16*dt + 4*(p & 3) .. +3, lane i
// ends up with dim 16*dt + i of rows 8*quad .. +3; a second read covers rows +4 .. +7.  No transposed copy of the
// tile is needed, in LDS or in memory.
template <int D>
__device__ inline bf16x8 lds_tr_operand(const bf16_t *tile, int dt) {
  const int p = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
  const int d0 = 16 * dt + 4 * (p & 3), seg = d0 >> 3, within = d0 & 7;
  const int row = 8 * quad + (p >> 2);
  const bf16_t *a0 = tile + TileGeom<D>::row_off(row, seg) + within;
  const bf16_t *a1 = tile + TileGeom<D>::row_off(row + 4, seg) + within;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a0);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a1);
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

// Cursor over the tiles of a list of key ranges held in LDS (rng_s/rng_e), uniform across the workgroup.  The end of
// the current range is kept in the cursor: LDS is read only when the walk moves to another range.
struct TileIter {
  int r, kb, end;
};
__device__ inline int lds_uniform(const int *p) { return __builtin_amdgcn_readfirstlane(*p); }
__device__ inline TileIter iter_begin(const int *rng_s, const int *rng_e, int nr) {
  TileIter it{0, 0, 0};
  if (nr > 0) {
    it.kb = lds_uniform(rng_s) & ~7;
    it.end = lds_uniform(rng_e);
  }
  return it;
}
__device__ inline TileIter iter_next(TileIter it, const int *rng_s, const int *rng_e, int nr, int step = 32) {
  it.kb += step;
  if (it.kb >= it.end) {
    ++it.r;
    if (it.r < nr) {
      it.kb = lds_uniform(rng_s + it.r) & ~7;
      it.end = lds_uniform(rng_e + it.r);
    }
  }
  return it;
}

// Workgroup -> (token tile, KV group).  Workgroups of a 1-D launch are dealt round-robin to the 8 XCDs, each with
// its own L2; this map keeps every XCD on ONE KV group and one contiguous run of token tiles, so the K/V rows it
// touches (one group's pooled keys, the windows and selected blocks of neighbouring tokens) stay L2 resident.
struct TileMap {
  int tile, g;
  bool valid;
};
__host__ __device__ inline int xcd_grid_size(int n_tiles, int Hkv) {
  if (Hkv > 8 || 8 % Hkv != 0) return n_tiles * Hkv;
  const int parts = 8 / Hkv;
  return 8 * ((n_tiles + parts - 1) / parts);
}
__device__ inline TileMap xcd_tile_map(int n_tiles, int Hkv) {
  const int L = blockIdx.x;
  if (Hkv > 8 || 8 % Hkv != 0) return TileMap{L % n_tiles, L / n_tiles, L < n_tiles * Hkv};
  const int xcd = L & 7, idx = L >> 3, parts = 8 / Hkv;
  const int g = xcd % Hkv, part = xcd / Hkv;
  const int tpp = (n_tiles + parts - 1) / parts;
  const int tile = part * tpp + idx;
  return TileMap{tile, g, idx < tpp && tile < n_tiles};
}

// The query rows of one wavefront: CB blocks of 16 columns; column n of block cb is workgroup row
// (wave*CB + cb)*16 + n = (token slot) * h_s + (head inside the group).
template <int D, int CB>
struct QRows {
  bf16x8 qop[CB][D / 32];
  int slot[CB], pos[CB], tok[CB], h[CB];
  bool valid[CB];
};

template <int D, int CB>
__device__ inline void load_rows(const bf16_t *Q, const MfmaView &v, int wg_pos0, int g, QRows<D, CB> &q) {
  const int wid = threadIdx.x >> 6, n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int row = (wid * CB + cb) * 16 + n;
    q.slot[cb] = row / v.hs;
    q.pos[cb] = wg_pos0 + q.slot[cb];
    q.valid[cb] = q.pos[cb] < v.N;
    q.tok[cb] = q.valid[cb] ? v.perm[q.pos[cb]] : 0;
    q.h[cb] = g * v.hs + row % v.hs;
    const bf16_t *src = Q + ((size_t)q.tok[cb] * v.Hq + q.h[cb]) * D + 8 * quad;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) q.qop[cb][ks] = q.valid[cb] ? ld8(src + 32 * ks) : zero8();
  }
}

// Running softmax state of CB blocks of 16 query columns (Algorithm 1's o, l, m), shared by the pipeline kernels and
// the block-centric selection kernel.
template <int D, int CB>
struct FwdState {
  f32x4 o[CB][D / 16];  // o[cb][dt][i]: output dim acc_dim(dt, quad) + i of query column n
  f32x4 l[CB];          // l[cb][0]: running sum of column n over all keys seen (the other three elements are unused)
  float m[CB];          // running max (raw score units)
};

template <int D, int CB>
__device__ inline void init_state(FwdState<D, CB> &st) {
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) st.o[cb][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    st.m[cb] = -INFINITY;
    st.l[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
}

// Walk the tiles of the key ranges rng_s/rng_e[0..nr) (LDS, workgroup-uniform).  Global loads run PF tiles (1 or 2)
// ahead of the tile being consumed, through PF register sets used alternately; LDS holds two stages: the stage
// written at step i is read at step i and overwritten at step i+2, with one barrier per step in between.
// enter(r) runs when the walk reaches range r, tile(stage, kb, r) consumes one staged tile.
// STEP: key rows consumed per step (32, or 64 when the tile set holds two consecutive 32-row tiles of one array).
template <int D, int NROW, int NTHR = 256, int PF = 2, int STEP = 32, class Enter, class Tile>
__device__ inline void run_pipeline(const TileSrc<NROW> &src, bf16_t *stage0, const int *rng_s, const int *rng_e, int nr,
                                    Enter enter, Tile tile) {
  using L = StageLayout<D, NROW>;
  if (nr > 0) {
    TileRegs<D, NROW, NTHR> regs[PF];
    TileIter cur = iter_begin(rng_s, rng_e, nr);
    TileIter ahead = cur;  // the last tile whose loads are in flight
    tile_load<D, NROW, NTHR>(regs[0], src, cur.kb);
    ahead = iter_next(cur, rng_s, rng_e, nr, STEP);
    if (ahead.r < nr) tile_load<D, NROW, NTHR>(regs[1], src, ahead.kb);
    int cur_r = -1;
    // register set 0 always feeds LDS stage 0 and set 1 stage 1 (the steps alternate), so the stage address is a
    // constant at each call site
    auto step = [&](TileRegs<D, NROW, NTHR> &r, int buf) {
      bf16_t *st = stage0 + buf * L::ELEMS;
      tile_store<D, NROW, NTHR>(r, st);
      // the request for the tile two steps ahead goes out while the LDS writes drain, before the barrier waits for them
      if (ahead.r < nr) ahead = iter_next(ahead, rng_s, rng_e, nr, STEP);
      if (ahead.r < nr) tile_load<D, NROW, NTHR>(r, src, ahead.kb);
      __syncthreads();
      if (cur.r != cur_r) {
        cur_r = cur.r;
        enter(cur_r);
      }
      tile(st, cur.kb, cur_r);
      cur = iter_next(cur, rng_s, rng_e, nr, STEP);
    };
    static_assert(PF == 2, "two register sets, two LDS stages");
    while (cur.r < nr) {
      step(regs[0], 0);
      if (!(cur.r < nr)) break;
      step(regs[1], 1);
    }
  }
  __syncthreads();
}

// Top-k over unsigned fixed-point scores S[0..n) held in LDS by one wavefront, ties to the lowest index, entirely in
// registers and wave ballots (no lane exchange, no LDS traffic inside the search).  Lane l keeps entries l, l+64, ...
// (up to R per lane, n <= 64*R).  The T-th largest value is found by building it bit by bit from the top: a
// candidate threshold is kept when at least T entries reach it (one compare + ballot + population count per
// register and bit).  Entries above the threshold are selected, entries equal to it in ascending index order until
// T are reached.  Writes T ids (base + index) in ascending order, padded with -1.
template <int R>
__device__ inline void topk_wave_bits(const uint32_t *S, int n, int T, int base, int32_t *out) {
  const int lane = threadIdx.x & 63;
  const uint64_t lt = (1ull << lane) - 1ull;
  uint32_t val[R];  // score + 1 (so that every real entry is >= 1); 0 marks "no entry"
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int j = r * 64 + lane;
    val[r] = j < n ? S[j] + 1u : 0u;
  }
  const int Tn = T < n ? T : n;
  uint32_t thr = 0u;
  if (Tn > 0) {
    for (int b = 31; b >= 0; --b) {
      const uint32_t cand = thr | (1u << b);
      int cnt = 0;
#pragma unroll
      for (int r = 0; r < R; ++r) cnt += __popcll(__ballot(val[r] >= cand));
      if (cnt >= Tn) thr = cand;
    }
  }
  int greater = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) greater += __popcll(__ballot(val[r] > thr));
  const int need = Tn - greater;  // entries equal to the threshold still to take, lowest indices first
  int written = 0, eq_before = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const bool eq = Tn > 0 && val[r] == thr;
    const uint64_t em = __ballot(eq);
    const bool sel = (Tn > 0 && val[r] > thr) || (eq && eq_before + (int)__popcll(em & lt) < need);
    eq_before += __popcll(em);
    const uint64_t sm = __ballot(sel);
    if (sel) out[written + __popcll(sm & lt)] = base + r * 64 + lane;
    written += __popcll(sm);
  }
  for (int w = written + lane; w < T; w += 64) out[w] = -1;
}

// Workgroup-wide [min lo, max hi) of the per-lane key ranges, and whether every row has exactly that range.
// scratch: 3 ints of LDS.  Returns through rs, re, uniform (all workgroup-uniform).
template <int CB>
__device__ inline void wg_range(int *scratch, const int (&lo)[CB], const int (&hi)[CB], const bool (&valid)[CB], int &rs,
                                int &re, bool &uniform) {
  if (threadIdx.x == 0) { scratch[0] = 0x7fffffff; scratch[1] = 0; scratch[2] = 1; }
  __syncthreads();
  int wlo = 0x7fffffff, whi = 0;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
    if (valid[cb]) { wlo = min(wlo, lo[cb]); whi = max(whi, hi[cb]); }
  wlo = wave_min_i(wlo);
  whi = wave_max_i(whi);
  if ((threadIdx.x & 63) == 0) { atomicMin(&scratch[0], wlo); atomicMax(&scratch[1], whi); }
  __syncthreads();
  rs = lds_uniform(&scratch[0]);
  re = lds_uniform(&scratch[1]);
  bool u = true;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) u = u && valid[cb] && lo[cb] == rs && hi[cb] == re;
  if (!__all(u) && (threadIdx.x & 63) == 0) scratch[2] = 0;
  __syncthreads();
  uniform = lds_uniform(&scratch[2]) != 0;
  if (re <= rs) { rs = 0; re = 0; }
}

// ---- top-k over unsigned fixed-point scores held in LDS by one wavefront (ties -> lowest id) ----
__device__ inline void topk_wave_u32(const uint32_t *S, int n, int T, int base, int32_t *out, uint32_t *sel) {
  const int lane = threadIdx.x & 63;
  const int words = (n + 31) >> 5;
  for (int i = lane; i < words; i += 64) sel[i] = 0u;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int rounds = T < n ? T : n;
  for (int r = 0; r < rounds; ++r) {
    uint64_t best = 0ull;
    for (int j = lane; j < n; j += 64) {
      if ((sel[j >> 5] >> (j & 31)) & 1u) continue;
      const uint64_t key = ((uint64_t)S[j] << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)j);
      best = key > best ? key : best;
    }
    best = wave_max_u64(best);
    const uint32_t j = 0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull);
    if (lane == 0) sel[j >> 5] |= 1u << (j & 31);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  int written = 0;
  for (int j0 = 0; j0 < n; j0 += 64) {
    const int j = j0 + lane;
    const bool s = j < n && ((sel[j >> 5] >> (j & 31)) & 1u);
    const uint64_t m = __ballot(s);
    if (s) out[written + __popcll(m & ((1ull << lane) - 1ull))] = base + j;
    written += __popcll(m);
  }
  for (int w = written + lane; w < T; w += 64) out[w] = -1;
}
