// bf16 MFMA backward kernels of SSA for gfx950.
//
// The paper states no backward pass; this is the softmax-attention gradient of eq. (2)-(4) with the selected
// index sets held constant, plus the gradient of the mean pool of eq. (5).  Per (query row, key) pair of a
// branch b with gate w_b:  P = exp(S - lse_b),  dP = <dO, V>,  dS = P (w_b dP - delta_b) scale,
// delta_b = w_b <dO, O_b>;  dV += w_b P dO,  dQ += dS K,  dK += dS Q.
//
// Three kernel families, all free of floating-point atomics (results do not depend on scheduling):
//   * m_bwd_dq: query-centric, same walk as the forward kernels (transposed scores, keys in the lanes), for the
//     compression and window branches;
//   * m_bwd_dq_bc: the selection branch's dQ, block-centric like its forward kernel (one partial dQ row per selected
//     block, added per token in rank order by m_dq_merge);
//   * m_bwd_dkv: key-centric; a wavefront owns 16*KB keys and streams the query rows that attend to them
//     (scores with the query rows in the lanes); the contractions over query rows take Q^T and dO^T from the
//     staged row-major tiles through the transposing LDS read.
#include "mfma_common.h"
#include "mfma_launch.h"
#include "mfma_qc.h"
#include "mfma_bc.h"
#include "profile.h"

#include <mutex>

namespace {

// ---------------------------------------------------------------------------------------------------------
// Pre-pass: dgates, per-row scalars in sorted order, sorted copies of Q and dO.
// One workgroup per sorted token position.
// ---------------------------------------------------------------------------------------------------------
struct PreArgs {
  const bf16_t *Q, *dO, *Ob, *gates;
  const float *lse;
  const int32_t *perm;
  int N, Hq, Hkv, hs, D;
  bf16_t *dgates;               // [N,Hq,3] caller order
  float *lse2s, *deltas, *gws;  // [3][N(pos)][Hq]
  float *deltag;                // [3][N(pos)][Hq]: delta taken over the rounded gate * dO rows (see below)
  bf16_t *Qs, *dOg;             // sorted row-major copies: Q [N(pos)][Hq][D], gate_b * dO [3][N(pos)][Hq][D]
};

__global__ __launch_bounds__(256) void m_bwd_pre(PreArgs a) {
  extern __shared__ bf16_t tile[];  // [Hq*D]: the token's dO rows
  const int pos = blockIdx.x, tok = a.perm[pos];
  const int HD = a.Hq * a.D;
  const size_t base = (size_t)tok * HD;
  bf16_t *td = tile;
  // The kernels that contract over dO rows of one branch (selection dQ, all dK/dV) take gate_b * dO: with it
  // dP_b = gate_b * (dO V^T) and dV_b = P^T (gate_b * dO) carry the gate of eq. (4) without any per-row multiplication.
  for (int e = threadIdx.x * 8; e < HD; e += blockDim.x * 8) {
    const bf16x8 xq = ld8(a.Q + base + e), xd = ld8(a.dO + base + e);
    *reinterpret_cast<bf16x8 *>(td + e) = xd;
    *reinterpret_cast<bf16x8 *>(a.Qs + (size_t)pos * HD + e) = xq;
    const bf16_t *gt = a.gates + ((size_t)tok * a.Hq + e / a.D) * 3;
#pragma unroll
    for (int b = 0; b < 3; ++b) {
      const float w = bf16_to_f32(gt[b]);
      bf16x8 y;
#pragma unroll
      for (int j = 0; j < 8; ++j) y[j] = (__bf16)(w * (float)xd[j]);
      *reinterpret_cast<bf16x8 *>(a.dOg + ((size_t)b * a.N + pos) * HD + e) = y;
    }
  }
  __syncthreads();
  // dgates and the row scalars: D/8 lanes per head (8 elements each), 256 / (D/8) heads per pass
  const int per = a.D / 8;  // 4, 8 or 16 lanes per head
  for (int h0 = 0; h0 < a.Hq; h0 += 256 / per) {
    const int h = h0 + threadIdx.x / per, part = threadIdx.x % per;
    // acc: <dO, O_b> (dgates, and delta_b = gate_b * it).  accg: <gate_b * dO as it was rounded into dOg, O_b>: the
    // kernels that read dOg subtract THIS delta from their dP, so that the two stay the same sum over the same numbers
    // (a softmax over one or two keys has dP = delta up to rounding, and dS = P (dP - delta) is what is left of it).
    float acc[3] = {0.f, 0.f, 0.f}, accg[3] = {0.f, 0.f, 0.f};
    if (h < a.Hq) {
      const bf16x8 go = *reinterpret_cast<const bf16x8 *>(td + h * a.D + 8 * part);
      const bf16_t *gt = a.gates + ((size_t)tok * a.Hq + h) * 3;
#pragma unroll
      for (int b = 0; b < 3; ++b) {
        const bf16x8 ob = ld8(a.Ob + (((size_t)b * a.N + tok) * a.Hq + h) * a.D + 8 * part);
        const float w = bf16_to_f32(gt[b]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          acc[b] += (float)go[j] * (float)ob[j];
          accg[b] += (float)(__bf16)(w * (float)go[j]) * (float)ob[j];
        }
      }
    }
    for (int off = 1; off < per; off <<= 1)
#pragma unroll
      for (int b = 0; b < 3; ++b) {
        acc[b] += __shfl_xor(acc[b], off);
        accg[b] += __shfl_xor(accg[b], off);
      }
    if (h < a.Hq && part < 3) {
      const int b = part;
      const float dot = b == 0 ? acc[0] : (b == 1 ? acc[1] : acc[2]);
      const size_t th = (size_t)tok * a.Hq + h;
      const float w = bf16_to_f32(a.gates[th * 3 + b]);
      a.dgates[th * 3 + b] = f32_to_bf16(dot);
      const size_t s = ((size_t)b * a.N + pos) * a.Hq + h;
      a.lse2s[s] = a.lse[((size_t)b * a.N + tok) * a.Hq + h] * LOG2E;
      a.deltas[s] = w * dot;
      a.gws[s] = w;
      a.deltag[s] = b == 0 ? accg[0] : (b == 1 ? accg[1] : accg[2]);
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// dQ: query-centric
// ---------------------------------------------------------------------------------------------------------
struct DqArgs {
  MfmaView v;
  const bf16_t *Q, *dO;
  const float *lse2s, *deltas, *gws;  // [3][N(pos)][Hq]
  float *dQp;  // [N(pos)][Hq][D] fp32: compression + window part of dQ
};

// One staged 32-key tile: transposed scores (K rows) and dP (V rows), then dQ^T += K^T dS^T (the K rows again, read
// through the transposing LDS load).  kt, vt: the staged K and V tiles, ln: the lane offsets of their operands (PTile).
// lse2 is +inf for a column whose token did not select the current block, which makes its P exactly zero.
template <int D, int CB, bool MASK>
__device__ inline void dq_tile(f32x4 (&acc)[CB][D / 16], const QRows<D, CB> &q, const bf16x8 (&dop)[CB][D / 32],
                               lds_cptr kt, lds_cptr vt, const typename PTile<D>::Lanes &ln, int kb, const int (&lo)[CB],
                               const int (&hi)[CB], const bool (&act)[CB], float sl2, float scale, const float (&lse2)[CB],
                               const float (&delta)[CB], const float (&gw)[CB]) {
  const int quad = threadIdx.x >> 4 & 3;
  float gws[CB], dls[CB];  // gate and delta with the softmax scale folded in: dS = P (gate dP - delta) scale
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) { gws[cb] = gw[cb] * scale; dls[cb] = delta[cb] * scale; }
  f32x4 s0[CB], s1[CB], p0[CB], p1[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) s0[cb] = s1[cb] = p0[cb] = p1[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    const bf16x8 k0 = p_row_operand<D>(kt, ln, 0, ks), k1 = p_row_operand<D>(kt, ln, 1, ks);
    const bf16x8 v0 = p_row_operand<D>(vt, ln, 0, ks), v1 = p_row_operand<D>(vt, ln, 1, ks);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      if (act[cb]) {
        s0[cb] = mfma16(k0, q.qop[cb][ks], s0[cb]);
        s1[cb] = mfma16(k1, q.qop[cb][ks], s1[cb]);
        p0[cb] = mfma16(v0, dop[cb][ks], p0[cb]);
        p1[cb] = mfma16(v1, dop[cb][ks], p1[cb]);
      }
  }
  bf16x8 dsb[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    if (!act[cb]) continue;
    const int rel = kb + 8 * quad - lo[cb];
    const unsigned len = (unsigned)(hi[cb] - lo[cb]);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float sv = j < 4 ? s0[cb][j & 3] : s1[cb][j & 3];
      const float dp = j < 4 ? p0[cb][j & 3] : p1[cb][j & 3];
      float p = fast_exp2(__builtin_fmaf(sv, sl2, -lse2[cb]));
      if (MASK && (unsigned)(rel + j) >= len) p = 0.f;  // lo <= key < hi as one unsigned comparison
      dsb[cb][j] = (__bf16)(p * __builtin_fmaf(gws[cb], dp, -dls[cb]));
    }
  }
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) {
    const bf16x8 ktd = p_tr_operand<D>(kt, ln, dt);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      if (act[cb]) acc[cb][dt] = mfma16(ktd, dsb[cb], acc[cb][dt]);
  }
}

// LDS plan of the dQ kernel (bytes): two stages (K rows, V rows) | 8 ints
template <int D>
__host__ __device__ inline size_t dq_lds_bytes() { return (size_t)2 * StageLayout<D, 2>::ELEMS * sizeof(bf16_t) + 32; }

// dQ of the compression branch, then of the (small) window branch, in the sorted token order; the sum is kept in fp32 by
// sorted position (dQp) for the merge with the selection branch's partials.
template <int D, int CB, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(D <= 64 && CB == 1 ? 4 : 2))) void m_bwd_dq(DqArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  using L = StageLayout<D, 2>;
  bf16_t *stage0 = (bf16_t *)smem;
  int *ints = (int *)(stage0 + 2 * L::ELEMS);
  const int quad = threadIdx.x >> 4 & 3;
  const int hs = a.v.hs, N = a.v.N, TW = NW * CB * 16 / hs;
  const TileMap tm = xcd_tile_map((N + TW - 1) / TW, a.v.Hkv);
  if (!tm.valid) return;
  const int g = tm.g, wg_pos0 = tm.tile * TW;
  QRows<D, CB> q;
  load_rows<D, CB>(a.Q, a.v, wg_pos0, g, q);
  bf16x8 dop[CB][D / 32];
  size_t rs_[CB];  // row of the per-row arrays, which are laid out by sorted position
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const bf16_t *src = a.dO + ((size_t)q.tok[cb] * a.v.Hq + q.h[cb]) * D + 8 * quad;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) dop[cb][ks] = q.valid[cb] ? ld8(src + 32 * ks) : zero8();
    rs_[cb] = (size_t)(q.valid[cb] ? q.pos[cb] : 0) * a.v.Hq + q.h[cb];
  }
  const size_t NH = (size_t)N * a.v.Hq;
  f32x4 acc[CB][D / 16];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) acc[cb][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const float sl2 = a.v.sl2, scale = a.v.scale;
  const size_t kstride = (size_t)a.v.Hkv * D;
  const typename PTile<D>::Lanes ln = PTile<D>::lanes();
  int lo[CB], hi[CB];
  bool act[CB];
  float lse2[CB], delta[CB], gw[CB];
  // one key range per branch, per-lane [lo, hi)
  for (int branch = 0; branch <= 2; branch += 2) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      if (branch == 0) {
        const int item = q.valid[cb] ? a.v.tok_item[q.pos[cb]] : 0;
        lo[cb] = q.valid[cb] ? a.v.cmp_batch[item] : 0;
        hi[cb] = q.valid[cb] ? a.v.cmp_batch[item + 1] : 0;
      } else {
        const int w = q.valid[cb] ? a.v.tok_win[q.pos[cb]] : 0;
        lo[cb] = q.valid[cb] ? a.v.win_start[w] : 0;
        hi[cb] = q.valid[cb] ? a.v.win_start[w + 1] : 0;
      }
      act[cb] = true;
      lse2[cb] = a.lse2s[branch * NH + rs_[cb]];
      delta[cb] = a.deltas[branch * NH + rs_[cb]];
      gw[cb] = a.gws[branch * NH + rs_[cb]];
    }
    int rs, re;
    bool uniform;
    wg_range<CB>(ints, lo, hi, q.valid, rs, re, uniform);
    if (threadIdx.x == 0) { ints[4] = rs; ints[5] = re; }
    __syncthreads();
    TileSrc<2> src = branch == 0
        ? TileSrc<2>{{a.v.Kc + (size_t)g * D, a.v.Vc + (size_t)g * D}, (uint32_t)kstride}
        : TileSrc<2>{{a.v.Ks + (size_t)g * D, a.v.Vs + (size_t)g * D}, (uint32_t)kstride};
    run_pipeline<D, 2, 64 * NW, 2>(
        src, stage0, ints + 4, ints + 5, re > rs ? 1 : 0, [](int) {},
        [&](const bf16_t *stg, int kb, int) {
          bf16_t *st = (bf16_t *)stg;
          if (uniform && kb >= rs && kb + 32 <= re)
            dq_tile<D, CB, false>(acc, q, dop, (lds_cptr)L::row_tile(st, 0), (lds_cptr)L::row_tile(st, 1), ln, kb, lo, hi, act, sl2,
                                  scale, lse2, delta, gw);
          else
            dq_tile<D, CB, true>(acc, q, dop, (lds_cptr)L::row_tile(st, 0), (lds_cptr)L::row_tile(st, 1), ln, kb, lo, hi, act, sl2,
                                 scale, lse2, delta, gw);
        });
  }
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    if (!q.valid[cb]) continue;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) *reinterpret_cast<f32x4 *>(a.dQp + rs_[cb] * D + acc_dim(dt, quad)) = acc[cb][dt];
  }
}

// ---------------------------------------------------------------------------------------------------------
// dK/dV: key-centric
// ---------------------------------------------------------------------------------------------------------
enum { DKV_WIN = 0, DKV_SLC = 1, DKV_CMP = 2 };

struct DkvArgs {
  MfmaView v;
  const bf16_t *Qs, *dOs;             // sorted copies [N(pos)][Hq][D]: Q, and the branch's gate * dO
  const float *lse2s, *deltas;        // already offset to the branch: [N(pos)][Hq]; delta over the rounded gate * dO rows
  const int32_t *sel_start, *sel_list;  // selection branch: query positions per (g, block)
  float *dK, *dV;                       // [rows][Hkv][D] fp32 (rows: sorted tokens, or compression blocks)
  const int32_t *chunk_start;           // selection branch: [Hkv*Ns+1] first work chunk of each (g, block)
  const int32_t *chunk_order;           // selection branch: execution order of the work chunks
  const int32_t *part_row_start;        // selection branch: [Hkv*Ns+1] first row of each (g, block)'s partial sums
  int chunk_len;                        // selection branch: query tokens per work chunk
  int tiles_per_block;                  // key tiles reserved per block in the grid
  int q_splits;                         // compression branch: query range split into this many parts
};

// LDS stage of the dK/dV kernels: ST tiles of 32 query rows each, of Q and of gate * dO (PTile layout: read both as
// they are and through the transposing LDS load), and two scalars per row: lse in log2 units and -delta.  The gate needs no
// scalar of its own: it rides on the dO rows, so dP = (gate dO) V^T and dV += P^T (gate dO) already carry it.
template <int D, int ST>
struct DkvStage {
  static constexpr int TILES_B = 2 * ST * PTile<D>::BYTES;  // Q tiles, then dO tiles
  static constexpr int BYTES = TILES_B + 2 * 32 * ST * 4;   // + [2][32*ST] floats
};

// A workgroup owns 16*KB*NW keys of one block (16*KB per wavefront, held in registers as MFMA B operands with their
// dK and dV accumulators) and streams the query rows that attend to them in stages of ST tiles of 32 rows (32/h_s
// token slots each), staged through LDS once per workgroup, double buffered, ONE barrier per stage: the loads of
// stage i+1 are in flight while stage i is consumed and land in the other buffer before the barrier.
template <int D, int KB, int MODE, int NW, int ST>
__global__ __launch_bounds__(64 * NW) void m_bwd_dkv(DkvArgs a) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int hs = a.v.hs, Hq = a.v.Hq;
  constexpr int WG_KEYS = 16 * KB * NW, NTHR = 64 * NW;
  using P = PTile<D>;
  using SG = DkvStage<D, ST>;
  int g = blockIdx.y, blk, tile;
  // key range of the block and query source
  int kbeg, kend, qbeg = 0, qend = 0;
  size_t out_row0 = 0;  // selection branch: first row of this chunk's partial sums
  const bf16_t *Kr, *Vr;
  if (MODE == DKV_WIN) {
    blk = blockIdx.x / a.tiles_per_block; tile = blockIdx.x % a.tiles_per_block;
    kbeg = a.v.win_start[blk]; kend = a.v.win_start[blk + 1];
    qbeg = kbeg; qend = kend;
    Kr = a.v.Ks; Vr = a.v.Vs;
  } else if (MODE == DKV_SLC) {
    // 1-D launch: the key tiles of one work chunk get workgroup ids 8 apart, i.e. they run on the same XCD close in
    // time, so the chunk's query rows are fetched into that L2 once.  Find the chunk's (g, block) by bisection over
    // the chunk prefix sums.
    const int per8 = 8 * a.tiles_per_block;
    const int nkeys = a.v.Hkv * a.v.Ns, wi = (int)(blockIdx.x / per8) * 8 + (int)(blockIdx.x % 8);
    int key, chunk;
    if (wi >= a.chunk_start[nkeys] || !bc_find_chunk(a.chunk_start, nkeys, a.chunk_order[wi], key, chunk)) return;
    g = key / a.v.Ns; blk = key % a.v.Ns; tile = (int)(blockIdx.x % per8) / 8;
    kbeg = a.v.slc_start[blk]; kend = a.v.slc_start[blk + 1];
    qbeg = a.sel_start[key] + chunk * a.chunk_len;
    qend = min(a.sel_start[key + 1], qbeg + a.chunk_len);
    out_row0 = (size_t)a.part_row_start[key] + (size_t)chunk * (kend - kbeg);
    Kr = a.v.Ks; Vr = a.v.Vs;
  } else {
    blk = blockIdx.x / a.tiles_per_block; tile = blockIdx.x % a.tiles_per_block;  // blk = batch item
    kbeg = a.v.cmp_batch[blk]; kend = a.v.cmp_batch[blk + 1];
    const int q0 = a.v.item_start[blk], q1 = a.v.item_start[blk + 1];
    const int per = (q1 - q0 + a.q_splits - 1) / a.q_splits;
    qbeg = min(q1, q0 + (int)blockIdx.z * per); qend = min(q1, qbeg + per);
    Kr = a.v.Kc; Vr = a.v.Vc;
  }
  if (kbeg + tile * WG_KEYS >= kend) return;             // whole workgroup beyond the block (uniform)
  const int k0 = kbeg + tile * WG_KEYS + wid * 16 * KB;  // this wave's first key
  const bool wave_on = k0 < kend;                        // idle wavefronts still help staging and keep the barriers
  const size_t kstride = (size_t)a.v.Hkv * D;
  // B operands: this wave's keys (column n of key block kbk), all of D (rows past the block are padded: in bounds)
  bf16x8 kop[KB][D / 32], vop[KB][D / 32];
#pragma unroll
  for (int kbk = 0; kbk < KB; ++kbk) {
    const size_t off = (size_t)(k0 + 16 * kbk + n) * kstride + (size_t)g * D + 8 * quad;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) {
      kop[kbk][ks] = ld8(Kr + off + 32 * ks);
      vop[kbk][ks] = ld8(Vr + off + 32 * ks);
    }
  }
  f32x4 dk[KB][D / 16], dv[KB][D / 16];
#pragma unroll
  for (int kbk = 0; kbk < KB; ++kbk)
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) dk[kbk][dt] = dv[kbk][dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  extern __shared__ __align__(16) unsigned char smem[];
  const int slots = 32 / hs;              // token slots per 32-row tile (hs divides 16)
  const int stage_slots = ST * slots;     // token slots per stage
  const float sl2 = a.v.sl2, scale = a.v.scale;
  const typename P::Lanes ln = P::lanes();
  // what this thread stages: NI 16-byte items of Q and of dO per stage, and (threads < 3*32*ST) one scalar
  constexpr int NI = (ST * P::ITEMS + NTHR - 1) / NTHR;
  int it_off[NI], it_slot[NI], it_col[NI];  // LDS byte offset, token slot inside the stage, element offset inside the token
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    // (when the stage has fewer items than the workgroup threads, the surplus threads repeat the last items)
    const int it = min((int)threadIdx.x + NTHR * i, ST * P::ITEMS - 1);
    const int rt = it / P::ITEMS, w = it % P::ITEMS, row = w / P::SEGS, seg = w % P::SEGS;
    it_off[i] = rt * P::BYTES + P::off(row, seg);
    it_slot[i] = rt * slots + row / hs;
    it_col[i] = (g * hs + row % hs) * D + seg * 8;
  }
  static_assert(2 * 32 * ST <= NTHR, "one scalar per thread and stage");
  const bool has_sc = threadIdx.x < 2 * 32 * ST;
  const int sc_arr = (threadIdx.x / (32 * ST)) & 1, sc_r = threadIdx.x % (32 * ST);
  const int sc_slot = (sc_r >> 5) * slots + (sc_r & 31) / hs, sc_head = g * hs + (sc_r & 31) % hs;
  const float *sc_src = sc_arr == 0 ? a.lse2s : a.deltas;
  const float sc_mul = sc_arr == 1 ? -1.0f : 1.0f;
  // sorted position of the token at list index li (-1: past the end)
  // (every load of the staging code is unconditional, with a clamped index: loads under a branch would make the
  // compiler wait for ALL outstanding loads at the next use instead of for the oldest ones)
  auto position = [&](int li) {
    const int v = MODE == DKV_SLC ? a.sel_list[min(li, qend - 1)] : li;
    return li < qend ? v : -1;
  };
  // One register set and two position sets: while stage i is consumed, the rows of stage i+1 are in flight (requested
  // right after the barrier, with the positions read during stage i-1) and the positions of stage i+2 are read.  One
  // stage of lookahead is enough because the chunks run in token order (the rows mostly come from the L2), and the
  // registers a second set would take are worth more to the tile code.  Nothing loaded is touched before the stage that
  // stores it into LDS.
  struct StageRegs { bf16x8 rq[NI], rd[NI]; float sc; bool missing; };
  struct StagePos { int it[NI], sc; };
  StageRegs regs;
  StagePos pos[2];
  auto load_positions = [&](int qb, StagePos &p) {
#pragma unroll
    for (int i = 0; i < NI; ++i) p.it[i] = position(qb + it_slot[i]);
    p.sc = position(qb + sc_slot);
  };
  auto load_stage = [&](StageRegs &r, const StagePos &p) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const uint32_t off = (uint32_t)max(p.it[i], 0) * (uint32_t)(Hq * D) + (uint32_t)it_col[i];
      r.rq[i] = ld8(a.Qs + off);
      r.rd[i] = ld8(a.dOs + off);
    }
    r.sc = sc_src[(uint32_t)max(p.sc, 0) * Hq + sc_head];  // (threads past the scalars load one they never store)
    r.missing = sc_arr == 0 && p.sc < 0;  // a missing row gets lse = +inf: it contributes exp2(-inf) = 0
  };
  auto store_stage = [&](const StageRegs &r, unsigned char *stage) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      *reinterpret_cast<bf16x8 *>(stage + it_off[i]) = r.rq[i];
      *reinterpret_cast<bf16x8 *>(stage + ST * P::BYTES + it_off[i]) = r.rd[i];
    }
    if (has_sc) ((float *)(stage + SG::TILES_B))[threadIdx.x] = r.missing ? INFINITY : r.sc * sc_mul;
  };

  load_positions(qbeg, pos[0]);
  load_positions(qbeg + stage_slots, pos[1]);
  load_stage(regs, pos[0]);
  int buf = 0;
  // stage qb: `regs` holds its rows; `p_rows` the positions of stage qb+1, `p_next` is refilled with those of stage qb+2
  auto do_stage = [&](int qb, const StagePos &p_rows, StagePos &p_next) {
    unsigned char *stage = smem + (size_t)buf * SG::BYTES;
    store_stage(regs, stage);
    __syncthreads();
    load_stage(regs, p_rows);                       // rows of the next stage; their positions were read one stage ago
    load_positions(qb + 2 * stage_slots, p_next);   // (past the end of the list: position -1, row 0 is loaded and dropped)
    buf ^= 1;
    if (!wave_on) return;
    const lds_cptr st0 = (lds_cptr)stage;
    const __attribute__((address_space(3))) float *scal =
        (const __attribute__((address_space(3))) float *)((lds_cptr)stage + SG::TILES_B) + 8 * quad;
#pragma unroll
    for (int rt = 0; rt < ST; ++rt) {
      // (row tiles past the end of the list are not skipped: their rows carry lse = +inf and add exact zeros, and a
      // stage without branches lets the tiles' matrix and vector work interleave)
      const lds_cptr Qt = st0 + rt * P::BYTES, Dt = st0 + (ST + rt) * P::BYTES;
      // this lane's eight consecutive query rows 8*quad .. +7 of the tile: row j is element j & 3 of sub-tile j >> 2
      float lse2[8], nd[8];  // lse (log2 units), -delta
      f32x4 s[KB][2], dp[KB][2];
      // dS = P (dP - delta) scale: the scale is applied once to the dK sums at the end.  With 32 keys per wavefront the
      // dP accumulators START from -delta of their rows, so the matrix instruction leaves dP - delta and dS costs one
      // multiplication per element; with 16 keys per wavefront (d = 128) the tile is too short to wait for the scalars
      // before its first matrix instruction, and -delta is added afterwards.
      constexpr bool DELTA_FIRST = KB > 1;
      {
        typedef const __attribute__((address_space(3))) f32x4 *f4p;
        const f32x4 l0 = *(f4p)(scal + 32 * rt), l1 = *(f4p)(scal + 32 * rt + 4);
        const f32x4 d0 = *(f4p)(scal + 32 * (ST + rt)), d1 = *(f4p)(scal + 32 * (ST + rt) + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          lse2[j] = l0[j]; lse2[4 + j] = l1[j];
          nd[j] = d0[j]; nd[4 + j] = d1[j];
        }
#pragma unroll
        for (int kbk = 0; kbk < KB; ++kbk) {
          s[kbk][0] = s[kbk][1] = f32x4{0.f, 0.f, 0.f, 0.f};
          dp[kbk][0] = DELTA_FIRST ? d0 : f32x4{0.f, 0.f, 0.f, 0.f};
          dp[kbk][1] = DELTA_FIRST ? d1 : f32x4{0.f, 0.f, 0.f, 0.f};
        }
      }
#pragma unroll
      for (int sa = 0; sa < 2; ++sa)
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
          const bf16x8 qa = p_row_operand<D>(Qt, ln, sa, ks), da = p_row_operand<D>(Dt, ln, sa, ks);
#pragma unroll
          for (int kbk = 0; kbk < KB; ++kbk) {
            s[kbk][sa] = mfma16(qa, kop[kbk][ks], s[kbk][sa]);
            dp[kbk][sa] = mfma16(da, vop[kbk][ks], dp[kbk][sa]);
          }
        }
      bf16x8 pw[KB], ds[KB];
#pragma unroll
      for (int kbk = 0; kbk < KB; ++kbk)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float sv = j < 4 ? s[kbk][0][j & 3] : s[kbk][1][j & 3];
          const float dpv = j < 4 ? dp[kbk][0][j & 3] : dp[kbk][1][j & 3];  // gate * dP (- delta)
          const float p = fast_exp2(__builtin_fmaf(sv, sl2, -lse2[j]));
          pw[kbk][j] = (__bf16)p;
          ds[kbk][j] = (__bf16)(p * (DELTA_FIRST ? dpv : dpv + nd[j]));
        }
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        const bf16x8 qt = p_tr_operand<D>(Qt, ln, dt), dot = p_tr_operand<D>(Dt, ln, dt);
#pragma unroll
        for (int kbk = 0; kbk < KB; ++kbk) {
          dv[kbk][dt] = mfma16(dot, pw[kbk], dv[kbk][dt]);
          dk[kbk][dt] = mfma16(qt, ds[kbk], dk[kbk][dt]);
        }
      }
    }
  };
  for (int qb = qbeg; qb < qend; qb += 2 * stage_slots) {
    do_stage(qb, pos[1], pos[0]);
    do_stage(qb + stage_slots, pos[0], pos[1]);  // (may lie wholly past the end: adds exact zeros; a branch here would
                                                 // cost a wait for all outstanding loads per iteration)
  }
  if (!wave_on) return;
  // --- store: lane holds dims acc_dim(dt, quad) + i of key column n
#pragma unroll
  for (int kbk = 0; kbk < KB; ++kbk) {
    const int key = k0 + 16 * kbk + n;
    if (key >= kend) continue;
    size_t off = ((size_t)key * a.v.Hkv + g) * D;
    if (MODE == DKV_CMP) off += (size_t)blockIdx.z * a.v.Nc * kstride;
    if (MODE == DKV_SLC) off = (out_row0 + (size_t)(key - kbeg)) * D;  // partial sums: [row][D]
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      *reinterpret_cast<float4 *>(a.dK + off + acc_dim(dt, quad)) =
          make_float4(dk[kbk][dt][0] * scale, dk[kbk][dt][1] * scale, dk[kbk][dt][2] * scale, dk[kbk][dt][3] * scale);
      *reinterpret_cast<float4 *>(a.dV + off + acc_dim(dt, quad)) =
          make_float4(dv[kbk][dt][0], dv[kbk][dt][1], dv[kbk][dt][2], dv[kbk][dt][3]);
    }
  }
}

// Selection branch: add the per-chunk partial sums of every key, in chunk order, onto the token-level gradients
// (which the window kernel wrote earlier on the same stream).  One thread per (sorted position, group, 4 dims).
__global__ void m_slc_reduce(const int32_t *__restrict__ tok_slc, const int32_t *__restrict__ slc_start,
                             const int32_t *__restrict__ chunk_start, const int32_t *__restrict__ part_row_start, int N,
                             int Hkv, int Ns, int D, const float *__restrict__ pK, const float *__restrict__ pV,
                             float *__restrict__ dKs, float *__restrict__ dVs) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per_row = D / 4;
  if (i >= (size_t)N * Hkv * per_row) return;
  const int d4 = (int)(i % per_row), g = (int)(i / per_row % Hkv), pos = (int)(i / ((size_t)per_row * Hkv));
  const int b = tok_slc[pos], key = g * Ns + b;
  const int klen = slc_start[b + 1] - slc_start[b], nch = chunk_start[key + 1] - chunk_start[key];
  const size_t row0 = (size_t)part_row_start[key] + (size_t)(pos - slc_start[b]);
  float4 sk = make_float4(0.f, 0.f, 0.f, 0.f), sv = sk;
  for (int c = 0; c < nch; ++c) {
    const size_t off = (row0 + (size_t)c * klen) * D + 4 * d4;
    const float4 ak = *reinterpret_cast<const float4 *>(pK + off), av = *reinterpret_cast<const float4 *>(pV + off);
    sk.x += ak.x; sk.y += ak.y; sk.z += ak.z; sk.w += ak.w;
    sv.x += av.x; sv.y += av.y; sv.z += av.z; sv.w += av.w;
  }
  const size_t dst = ((size_t)pos * Hkv + g) * D + 4 * d4;
  float4 ck = *reinterpret_cast<float4 *>(dKs + dst), cv = *reinterpret_cast<float4 *>(dVs + dst);
  ck.x += sk.x; ck.y += sk.y; ck.z += sk.z; ck.w += sk.w;
  cv.x += sv.x; cv.y += sv.y; cv.z += sv.z; cv.w += sv.w;
  *reinterpret_cast<float4 *>(dKs + dst) = ck;
  *reinterpret_cast<float4 *>(dVs + dst) = cv;
}

// ---------------------------------------------------------------------------------------------------------
// Finish: dK[tok] = dKs[pos] + (sum over query splits of dKc[c]) / count(c)  (gradient of the mean pool),
// scattered back to caller order.  One workgroup per compression block.  With dKc_out/dVc_out given (the pooled
// rows were the caller's), the summed block gradients go there instead and dK, dV keep the token-level part only.
// ---------------------------------------------------------------------------------------------------------
__global__ void m_bwd_finish(const int32_t *__restrict__ perm, const int32_t *__restrict__ cmp_start, int Nc, int row,
                             int splits, const float *__restrict__ dKs, const float *__restrict__ dVs,
                             const float *__restrict__ dKc, const float *__restrict__ dVc, bf16_t *__restrict__ dK,
                             bf16_t *__restrict__ dV, float *__restrict__ dKc_out, float *__restrict__ dVc_out) {
  const int c = blockIdx.x;
  const int b = cmp_start[c], e = cmp_start[c + 1];
  const float inv = 1.0f / (float)(e - b);
  for (int f = threadIdx.x; f < row; f += blockDim.x) {
    float ck = 0.f, cv = 0.f;
    for (int s = 0; s < splits; ++s) {
      ck += dKc[((size_t)s * Nc + c) * row + f];
      cv += dVc[((size_t)s * Nc + c) * row + f];
    }
    if (dKc_out) {
      dKc_out[(size_t)c * row + f] = ck;
      dVc_out[(size_t)c * row + f] = cv;
      ck = cv = 0.f;
    }
    ck *= inv;
    cv *= inv;
    for (int pos = b; pos < e; ++pos) {
      const size_t dst = (size_t)perm[pos] * row + f;
      dK[dst] = f32_to_bf16(dKs[(size_t)pos * row + f] + ck);
      dV[dst] = f32_to_bf16(dVs[(size_t)pos * row + f] + cv);
    }
  }
}

// Shape of the block-centric selection dQ kernel per head dimension: wavefronts per workgroup, keys held in LDS at a time.
// 16-column blocks per wavefront of the compression + window dQ kernel: with two, every K and V operand read from LDS
// feeds two matrix instructions (202 registers, two waves per SIMD; 1.15 -> 1.09 ms at the benchmark shape); head_dim
// 128 keeps one (its accumulators alone would double).
template <int D> constexpr int dq_cb() { return D <= 64 ? 2 : 1; }
constexpr int KB_KEYS_MAX = 2;  // key blocks of 16 per wavefront in the dK/dV kernels (1 at head_dim 128: registers)
// wavefronts per workgroup there (16*KB_KEYS keys each): blocks and windows hold ~130 tokens, an item's pooled keys
// thousands, so the compression branch takes wider workgroups (fewer passes over the query rows)
template <int D> struct DkvWaves { static constexpr int N = 4; };
template <> struct DkvWaves<128> { static constexpr int N = 8; };  // 16 keys per wavefront there: 128 keys per workgroup again
// 32-row tiles of query rows per LDS stage (one barrier per stage)
template <int D> struct DkvShape { static constexpr int ST = 2; };

template <int D>
int launch_backward(const MfmaView &v, const BwdBuffers &w, const void *q, const void *gates, const void *out_branch,
                    const float *lse, const int32_t *idx, const void *dout, void *dq, void *dk, void *dv, void *dgates,
                    const ssa_blocks *blk, int B, hipStream_t s) {
  const int N = v.N, Hq = v.Hq, Hkv = v.Hkv, row = Hkv * D;
  const size_t NH = (size_t)N * Hq;
  {
    ProfScope ps(PROF_BWD_PRE, s);
    PreArgs a{(const bf16_t *)q, (const bf16_t *)dout, (const bf16_t *)out_branch, (const bf16_t *)gates, lse, v.perm,
              N, Hq, Hkv, v.hs, D, (bf16_t *)dgates, w.lse2s, w.deltas, w.gws, w.deltag, w.Qs, w.dOg};
    m_bwd_pre<<<N, 256, (size_t)Hq * D * sizeof(bf16_t), s>>>(a);
  }
  static std::once_flag dq_once;  // raise the dynamic LDS limit once per process for this instantiation
  std::call_once(dq_once, [] {
    (void)hipFuncSetAttribute((const void *)m_bwd_dq<D, dq_cb<D>(), 4>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  });
  {
    ProfScope ps0(PROF_BWD_DQ_CMP, s);
    DqArgs a{v, (const bf16_t *)q, (const bf16_t *)dout, w.lse2s, w.deltas, w.gws, w.dQp};
    constexpr int CB = dq_cb<D>(), NW0 = 4;
    const int tw0 = NW0 * CB * 16 / v.hs;
    m_bwd_dq<D, CB, NW0><<<dim3(xcd_grid_size((N + tw0 - 1) / tw0, Hkv)), 64 * NW0, dq_lds_bytes<D>(), s>>>(a);
  }
  {
    ProfScope ps(PROF_BWD_INVERT, s);
    const int rc = sel_index_build(idx, v.perm, v.slc_start, N, Hkv, v.T, v.Ns, w.sel, true, s);
    if (rc != SSA_OK) return rc;
  }
  {
    ProfScope ps1(PROF_BWD_DQ, s);
    const int rc = slc_dq_kernel(v, D, w, idx, s);
    if (rc != SSA_OK) return rc;
  }
  {
    ProfScope ps2(PROF_BWD_DQ_MERGE, s);
    const int rc = slc_dq_merge_kernel(v, D, w, idx, dq, s);
    if (rc != SSA_OK) return rc;
  }
  constexpr int KB_KEYS = D >= 128 ? 1 : KB_KEYS_MAX;
  constexpr int DKV_WAVES = DkvWaves<D>::N, DKV_WAVES_CMP = DkvWaves<D>::N;
  constexpr int WG_KEYS = 16 * KB_KEYS * DKV_WAVES, WG_KEYS_CMP = 16 * KB_KEYS * DKV_WAVES_CMP;
  static_assert(WG_KEYS <= SSA_KEY_PAD && WG_KEYS_CMP <= SSA_KEY_PAD, "key tiles may read up to WG_KEYS rows past a block");
  constexpr int ST = DkvShape<D>::ST;
  const size_t dkv_lds = (size_t)2 * DkvStage<D, ST>::BYTES;
  static std::once_flag dkv_once;
  std::call_once(dkv_once, [] {
    (void)hipFuncSetAttribute((const void *)m_bwd_dkv<D, KB_KEYS, DKV_WIN, DKV_WAVES, ST>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    (void)hipFuncSetAttribute((const void *)m_bwd_dkv<D, KB_KEYS, DKV_SLC, DKV_WAVES, ST>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    (void)hipFuncSetAttribute((const void *)m_bwd_dkv<D, KB_KEYS, DKV_CMP, DKV_WAVES_CMP, ST>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  });
  DkvArgs base{v, w.Qs, nullptr, nullptr, nullptr, w.sel.start, w.sel.list,
               w.dKs, w.dVs, w.sel.chunk_start, w.sel.order, w.sel.part_row_start, w.sel.chunk_len, 1, 1};
  {
    ProfScope ps(PROF_BWD_DKV_WIN, s);
    DkvArgs a = base;
    a.lse2s = w.lse2s + 2 * NH; a.deltas = w.deltag + 2 * NH; a.dOs = w.dOg + 2 * NH * D;
    a.tiles_per_block = (blk->win_tok_max + WG_KEYS - 1) / WG_KEYS;
    m_bwd_dkv<D, KB_KEYS, DKV_WIN, DKV_WAVES, ST><<<dim3(blk->Nw * a.tiles_per_block, Hkv), 64 * DKV_WAVES, dkv_lds, s>>>(a);
  }
  {
    ProfScope ps(PROF_BWD_DKV_SLC, s);
    DkvArgs a = base;
    a.lse2s = w.lse2s + NH; a.deltas = w.deltag + NH; a.dOs = w.dOg + NH * D;
    a.dK = w.pK; a.dV = w.pV;
    a.tiles_per_block = (blk->slc_tok_max + WG_KEYS - 1) / WG_KEYS;
    m_bwd_dkv<D, KB_KEYS, DKV_SLC, DKV_WAVES, ST><<<dim3((w.max_chunks + 7) / 8 * 8 * a.tiles_per_block), 64 * DKV_WAVES, dkv_lds, s>>>(a);
    const size_t items = (size_t)N * Hkv * (D / 4);
    m_slc_reduce<<<(unsigned)((items + 255) / 256), 256, 0, s>>>(blk->tok_slc, v.slc_start, w.sel.chunk_start, w.sel.part_row_start, N,
                                                                 Hkv, v.Ns, D, w.pK, w.pV, w.dKs, w.dVs);
  }
  {
    ProfScope ps(PROF_BWD_DKV_CMP, s);
    DkvArgs a = base;
    a.lse2s = w.lse2s; a.deltas = w.deltag; a.dOs = w.dOg;
    a.dK = w.dKc; a.dV = w.dVc;
    a.tiles_per_block = (blk->c_max + WG_KEYS_CMP - 1) / WG_KEYS_CMP;
    a.q_splits = w.q_splits;
    m_bwd_dkv<D, KB_KEYS, DKV_CMP, DKV_WAVES_CMP, ST><<<dim3(B * a.tiles_per_block, Hkv, w.q_splits), 64 * DKV_WAVES_CMP, dkv_lds, s>>>(a);
  }
  {
    ProfScope ps(PROF_BWD_FINISH, s);
    m_bwd_finish<<<v.Nc, 128, 0, s>>>(v.perm, v.cmp_start, v.Nc, row, w.q_splits, w.dKs, w.dVs, w.dKc, w.dVc, (bf16_t *)dk,
                                      (bf16_t *)dv, w.dKc_out, w.dVc_out);
  }
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

}  // namespace

int mfma_backward_kernels(const MfmaView &v, int D, const BwdBuffers &w, const void *q, const void *gates,
                          const void *out_branch, const float *lse, const int32_t *idx, const void *dout, void *dq,
                          void *dk, void *dv, void *dgates, const ssa_blocks *blk, int B, hipStream_t s) {
  switch (D) {
    case 32: return launch_backward<32>(v, w, q, gates, out_branch, lse, idx, dout, dq, dk, dv, dgates, blk, B, s);
    case 64: return launch_backward<64>(v, w, q, gates, out_branch, lse, idx, dout, dq, dk, dv, dgates, blk, B, s);
    case 128: return launch_backward<128>(v, w, q, gates, out_branch, lse, idx, dout, dq, dk, dv, dgates, blk, B, s);
    default: return SSA_ERR_UNSUPPORTED;
  }
}
