// bf16 MFMA backward kernels of SSA for gfx950.
//
// The paper states no backward pass; this is the softmax-attention gradient of eq. (2)-(4) with the selected
// index sets held constant, plus the gradient of the mean pool of eq. (5).  Per (query row, key) pair of a
// branch b with gate w_b:  P = exp(S - lse_b),  dP = <dO, V>,  dS = P (w_b dP - delta_b) scale,
// delta_b = w_b <dO, O_b>;  dV += w_b P dO,  dQ += dS K,  dK += dS Q.
//
// Two kernel families, both free of floating-point atomics (results do not depend on scheduling):
//   * m_bwd_dq: query-centric, same walk as the forward kernels (transposed scores, keys in the lanes);
//   * m_bwd_dkv: key-centric; a wavefront owns 16*KB keys and streams the query rows that attend to them
//     (scores with the query rows in the lanes); the contractions over query rows take Q^T and dO^T from the
//     staged row-major tiles through the transposing LDS read.
#include "mfma_common.h"
#include "mfma_launch.h"
#include "mfma_qc.h"
#include "profile.h"

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
  bf16_t *Qs, *dOs;             // [N(pos)][Hq][D] sorted row-major copies
};

__global__ __launch_bounds__(256) void m_bwd_pre(PreArgs a) {
  extern __shared__ bf16_t tile[];  // [Hq*D]: the token's dO rows
  const int pos = blockIdx.x, tok = a.perm[pos];
  const int HD = a.Hq * a.D;
  const size_t base = (size_t)tok * HD;
  bf16_t *td = tile;
  for (int e = threadIdx.x * 8; e < HD; e += blockDim.x * 8) {
    const bf16x8 xq = ld8(a.Q + base + e), xd = ld8(a.dO + base + e);
    *reinterpret_cast<bf16x8 *>(td + e) = xd;
    *reinterpret_cast<bf16x8 *>(a.Qs + (size_t)pos * HD + e) = xq;
    *reinterpret_cast<bf16x8 *>(a.dOs + (size_t)pos * HD + e) = xd;
  }
  __syncthreads();
  // dgates and the row scalars: D/8 lanes per head (8 elements each), 256 / (D/8) heads per pass
  const int per = a.D / 8;  // 4, 8 or 16 lanes per head
  for (int h0 = 0; h0 < a.Hq; h0 += 256 / per) {
    const int h = h0 + threadIdx.x / per, part = threadIdx.x % per;
    float acc[3] = {0.f, 0.f, 0.f};
    if (h < a.Hq) {
      const bf16x8 go = *reinterpret_cast<const bf16x8 *>(td + h * a.D + 8 * part);
#pragma unroll
      for (int b = 0; b < 3; ++b) {
        const bf16x8 ob = ld8(a.Ob + (((size_t)b * a.N + tok) * a.Hq + h) * a.D + 8 * part);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[b] += (float)go[j] * (float)ob[j];
      }
    }
    for (int off = 1; off < per; off <<= 1)
#pragma unroll
      for (int b = 0; b < 3; ++b) acc[b] += __shfl_xor(acc[b], off);
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
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// dQ: query-centric
// ---------------------------------------------------------------------------------------------------------
struct DqArgs {
  MfmaView v;
  const bf16_t *Q, *dO;
  const int32_t *idx;
  const float *lse2s, *deltas, *gws;  // [3][N(pos)][Hq]
  bf16_t *dQ;
  float *dQp;  // [N(pos)][Hq][D] fp32: compression + window part of dQ, handed from the first dQ kernel to the second
  const int32_t *slc_order;  // [Hkv][N] token order of the selection part (caller indices), or NULL: sorted order
  const int32_t *inv_perm;   // [N] caller index -> sorted position
};

// One staged 32-key tile: transposed scores (K rows) and dP (V rows), then dQ^T += K^T dS^T (the K rows again, read
// through the transposing LDS load).
// lse2 is +inf for a column whose token did not select the current block, which makes its P exactly zero.
template <int D, int CB, bool MASK>
__device__ inline void dq_tile(f32x4 (&acc)[CB][D / 16], const QRows<D, CB> &q, const bf16x8 (&dop)[CB][D / 32],
                               const bf16_t *ktile, const bf16_t *vtile, int kb, const int (&lo)[CB],
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
    const bf16x8 k0 = lds_row_operand<D>(ktile, 0, ks), k1 = lds_row_operand<D>(ktile, 1, ks);
    const bf16x8 v0 = lds_row_operand<D>(vtile, 0, ks), v1 = lds_row_operand<D>(vtile, 1, ks);
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
    const bf16x8 kt = lds_tr_operand<D>(ktile, dt);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      if (act[cb]) acc[cb][dt] = mfma16(kt, dsb[cb], acc[cb][dt]);
  }
}

// LDS plan of the dQ kernel (bytes): two stages (K rows, V rows) | 8 ints | selection lists as in the
// forward selection kernel.
template <int D>
__host__ __device__ inline size_t dq_lds_bytes(int tw, int T, int Ns) {
  return (size_t)2 * StageLayout<D, 2>::ELEMS * sizeof(bf16_t) + 32 + ((size_t)tw * T * 4 + (size_t)(Ns + 31) / 32 + 4) * 4;
}

// PART 0: compression branch, then the (small) window branch, in the sorted token order; result kept in fp32.
// PART 1: selection branch on top of it, in the selection order of the KV head (tokens with similar selected sets
// next to each other), final bf16 dQ.
template <int D, int CB, int PART, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(D <= 64 ? 4 : 2))) void m_bwd_dq(DqArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  using L = StageLayout<D, 2>;
  bf16_t *stage0 = (bf16_t *)smem;
  int *ints = (int *)(stage0 + 2 * L::ELEMS);
  const int quad = threadIdx.x >> 4 & 3;
  const int hs = a.v.hs, T = a.v.T, N = a.v.N, TW = NW * CB * 16 / hs;
  const TileMap tm = xcd_tile_map((N + TW - 1) / TW, a.v.Hkv);
  if (!tm.valid) return;
  const int g = tm.g, wg_pos0 = tm.tile * TW;
  int *Irows = ints + 8;
  int *ub = Irows + TW * T, *us = ub + TW * T, *ue = us + TW * T;
  uint32_t *bits = (uint32_t *)(ue + TW * T);
  QRows<D, CB> q;
  MfmaView vo = a.v;  // position -> token: the sorted order, or the selection order of this KV head
  const bool reordered = PART == 1 && a.slc_order != nullptr;
  if (reordered) vo.perm = a.slc_order + (size_t)g * N;
  load_rows<D, CB>(a.Q, vo, wg_pos0, g, q);
  bf16x8 dop[CB][D / 32];
  size_t rs_[CB];  // row of the per-row arrays, which are laid out by sorted position
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const bf16_t *src = a.dO + ((size_t)q.tok[cb] * a.v.Hq + q.h[cb]) * D + 8 * quad;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) dop[cb][ks] = q.valid[cb] ? ld8(src + 32 * ks) : zero8();
    const int spos = !q.valid[cb] ? 0 : (reordered ? a.inv_perm[q.tok[cb]] : q.pos[cb]);
    rs_[cb] = (size_t)spos * a.v.Hq + q.h[cb];
  }
  const size_t NH = (size_t)N * a.v.Hq;
  f32x4 acc[CB][D / 16];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      acc[cb][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (PART == 1 && q.valid[cb])
        acc[cb][dt] = *reinterpret_cast<const f32x4 *>(a.dQp + rs_[cb] * D + 16 * dt + 4 * quad);
    }
  const float sl2 = a.v.sl2, scale = a.v.scale;
  const size_t kstride = (size_t)a.v.Hkv * D;
  int lo[CB], hi[CB];
  bool act[CB];
  float lse2[CB], delta[CB], gw[CB];

  // ---- compression and window branches: one key range each, per-lane [lo, hi)
  for (int branch = 0; PART == 0 && branch <= 2; branch += 2) {
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
            dq_tile<D, CB, false>(acc, q, dop, L::row_tile(st, 0), L::row_tile(st, 1), kb, lo, hi, act, sl2,
                                  scale, lse2, delta, gw);
          else
            dq_tile<D, CB, true>(acc, q, dop, L::row_tile(st, 0), L::row_tile(st, 1), kb, lo, hi, act, sl2,
                                 scale, lse2, delta, gw);
        });
  }
  // ---- selection branch: union of the selected blocks of the workgroup's tokens
  if (PART == 1) {
    build_union(vo, a.idx, wg_pos0, g, TW, Irows, ub, us, ue, bits, &ints[0]);
    const int nr = lds_uniform(&ints[0]);
    int jc[CB];
    float lse_own[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      jc[cb] = 0; lo[cb] = hi[cb] = 0; act[cb] = false;
      lse_own[cb] = a.lse2s[NH + rs_[cb]];
      delta[cb] = a.deltas[NH + rs_[cb]];
      gw[cb] = a.gws[NH + rs_[cb]];
    }
    int rs = 0, re = 0;
    TileSrc<2> src{{a.v.Ks + (size_t)g * D, a.v.Vs + (size_t)g * D}, (uint32_t)kstride};
    run_pipeline<D, 2, 64 * NW, 1>(
        src, stage0, us, ue, nr,
        [&](int r) {
          const int b = lds_uniform(&ub[r]);
          rs = lds_uniform(&us[r]);
          re = lds_uniform(&ue[r]);
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) {
            const int cur = (q.valid[cb] && jc[cb] < T) ? Irows[q.slot[cb] * T + jc[cb]] : -1;
            const bool sel = cur == b;
            if (sel) ++jc[cb];
            lo[cb] = sel ? rs : 0;
            hi[cb] = sel ? re : 0;
            lse2[cb] = sel ? lse_own[cb] : INFINITY;
            act[cb] = __any(sel);
          }
        },
        [&](const bf16_t *stg, int kb, int) {
          bool any = false;
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) any = any || act[cb];
          if (!any) return;
          bf16_t *st = (bf16_t *)stg;
          if (kb >= rs && kb + 32 <= re)
            dq_tile<D, CB, false>(acc, q, dop, L::row_tile(st, 0), L::row_tile(st, 1), kb, lo, hi, act, sl2,
                                  scale, lse2, delta, gw);
          else
            dq_tile<D, CB, true>(acc, q, dop, L::row_tile(st, 0), L::row_tile(st, 1), kb, lo, hi, act, sl2,
                                 scale, lse2, delta, gw);
        });
  }
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    if (!q.valid[cb]) continue;
    if (PART == 0) {
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) *reinterpret_cast<f32x4 *>(a.dQp + rs_[cb] * D + 16 * dt + 4 * quad) = acc[cb][dt];
      continue;
    }
    bf16_t *o = a.dQ + ((size_t)q.tok[cb] * a.v.Hq + q.h[cb]) * D + 4 * quad;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      bf16x4 w;
#pragma unroll
      for (int i = 0; i < 4; ++i) w[i] = (__bf16)acc[cb][dt][i];
      *reinterpret_cast<bf16x4 *>(o + 16 * dt) = w;
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// dK/dV: key-centric
// ---------------------------------------------------------------------------------------------------------
enum { DKV_WIN = 0, DKV_SLC = 1, DKV_CMP = 2 };

struct DkvArgs {
  MfmaView v;
  const bf16_t *Qs, *dOs;             // sorted copies: [N(pos)][Hq][D]
  const float *lse2s, *deltas, *gws;  // already offset to the branch: [N(pos)][Hq]
  const int32_t *sel_start, *sel_list;  // selection branch: query positions per (g, block)
  float *dK, *dV;                       // [rows][Hkv][D] fp32 (rows: sorted tokens, or compression blocks)
  const int32_t *chunk_start;           // selection branch: [Hkv*Ns+1] first work chunk of each (g, block)
  const int32_t *part_row_start;        // selection branch: [Hkv*Ns+1] first row of each (g, block)'s partial sums
  int chunk_len;                        // selection branch: query tokens per work chunk
  int tiles_per_block;                  // key tiles reserved per block in the grid
  int q_splits;                         // compression branch: query range split into this many parts
};

// LDS stage of the dK/dV kernels: 32 query rows as row-major tiles of Q and dO (read both as they are and through
// the transposing LDS load), and the rows' scalars (lse in log2 units, delta, gate).
template <int D>
struct DkvStage {
  using G = TileGeom<D>;
  static constexpr int ELEMS = 2 * G::ROW_ELEMS;
  static constexpr int BYTES = ELEMS * 2 + 3 * 32 * 4;
};

// A workgroup owns 64*KB keys of one block (16*KB per wavefront, held in registers as MFMA B operands) and
// streams the query rows that attend to them in tiles of 32 rows = 32/h_s token slots, staged through LDS once per
// workgroup and double buffered.
template <int D, int KB, int MODE, int NW>
__global__ __launch_bounds__(64 * NW) void m_bwd_dkv(DkvArgs a) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int hs = a.v.hs, Hq = a.v.Hq;
  constexpr int WG_KEYS = 16 * KB * NW, NTHR = 64 * NW;
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
    const int nkeys = a.v.Hkv * a.v.Ns, w = (int)(blockIdx.x / per8) * 8 + (int)(blockIdx.x % 8);
    if (w >= a.chunk_start[nkeys]) return;
    int lo = 0, hi = nkeys;  // chunk_start[lo] <= w < chunk_start[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (a.chunk_start[mid] <= w) lo = mid; else hi = mid;
    }
    const int key = lo, chunk = w - a.chunk_start[key];
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
  using G = TileGeom<D>;
  using SG = DkvStage<D>;
  const int slots = 32 / hs;  // token slots per 32-row tile (hs is 8 or 16)
  const float sl2 = a.v.sl2, scale = a.v.scale;
  // sorted positions of the token slots of the tile that starts at list index qb (-1: past the end)
  auto positions = [&](int qb, int (&p)[4]) {
#pragma unroll
    for (int sidx = 0; sidx < 4; ++sidx) {
      const int sl = qb + sidx;
      p[sidx] = (sidx < slots && sl < qend) ? (MODE == DKV_SLC ? a.sel_list[sl] : sl) : -1;
    }
  };
  bf16x8 rq[G::row_per_thread(NTHR)], rd[G::row_per_thread(NTHR)];
  float sc = 0.f;
  auto pick = [](const int (&p)[4], int i) { return i == 0 ? p[0] : (i == 1 ? p[1] : (i == 2 ? p[2] : p[3])); };
  auto load_tile = [&](const int (&p)[4]) {
#pragma unroll
    for (int i = 0; i < G::row_per_thread(NTHR); ++i) {
      const int it = threadIdx.x + NTHR * i;
      if (G::ROW_ITEMS % NTHR == 0 || it < G::ROW_ITEMS) {
        const int row = it / (D / 8), seg = it % (D / 8);
        const int pos = max(pick(p, row / hs), 0);
        const uint32_t off = ((uint32_t)pos * Hq + g * hs + row % hs) * D + seg * 8;
        rq[i] = ld8(a.Qs + off);
        rd[i] = ld8(a.dOs + off);
      }
    }
    if (threadIdx.x < 96) {
      const int arr = threadIdx.x >> 5, row = threadIdx.x & 31;
      const int pos = pick(p, row / hs);
      const uint32_t rsx = (uint32_t)max(pos, 0) * Hq + g * hs + row % hs;
      const float *srcp = arr == 0 ? a.lse2s : (arr == 1 ? a.deltas : a.gws);
      sc = srcp[rsx];
      if (arr == 0 && pos < 0) sc = INFINITY;  // a missing row contributes exp2(-inf) = 0
    }
  };
  auto store_tile = [&](unsigned char *stage) {
    bf16_t *e = (bf16_t *)stage;
#pragma unroll
    for (int i = 0; i < G::row_per_thread(NTHR); ++i) {
      const int it = threadIdx.x + NTHR * i;
      if (G::ROW_ITEMS % NTHR == 0 || it < G::ROW_ITEMS) {
        const int off = G::row_off(it / (D / 8), it % (D / 8));
        *reinterpret_cast<bf16x8 *>(e + off) = rq[i];
        *reinterpret_cast<bf16x8 *>(e + G::ROW_ELEMS + off) = rd[i];
      }
    }
    if (threadIdx.x < 96) ((float *)(stage + SG::ELEMS * 2))[threadIdx.x] = sc;
  };

  int pcur[4], pnxt[4];
  positions(qbeg, pcur);
  if (qbeg < qend) load_tile(pcur);
  positions(qbeg + slots, pnxt);
  int buf = 0;
  for (int qb = qbeg; qb < qend; qb += slots) {
    unsigned char *stage = smem + (size_t)buf * SG::BYTES;
    store_tile(stage);
    __syncthreads();
    if (qb + slots < qend) {
      load_tile(pnxt);
      positions(qb + 2 * slots, pnxt);
    }
    buf ^= 1;
    if (!wave_on) continue;
    const bf16_t *Qr = (const bf16_t *)stage, *Dr = Qr + G::ROW_ELEMS;
    const float *scal = (const float *)(stage + SG::ELEMS * 2);
    f32x4 s[KB][2], dp[KB][2];
#pragma unroll
    for (int kbk = 0; kbk < KB; ++kbk)
#pragma unroll
      for (int sa = 0; sa < 2; ++sa) s[kbk][sa] = dp[kbk][sa] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sa = 0; sa < 2; ++sa)
#pragma unroll
      for (int ks = 0; ks < D / 32; ++ks) {
        const bf16x8 qa = lds_row_operand<D>(Qr, sa, ks), da = lds_row_operand<D>(Dr, sa, ks);
#pragma unroll
        for (int kbk = 0; kbk < KB; ++kbk) {
          s[kbk][sa] = mfma16(qa, kop[kbk][ks], s[kbk][sa]);
          dp[kbk][sa] = mfma16(da, vop[kbk][ks], dp[kbk][sa]);
        }
      }
    // this lane's eight consecutive query rows 8*quad .. +7
    float lse2[8], delta[8], gw[8];
    {
      const float4 l0 = *reinterpret_cast<const float4 *>(scal + 8 * quad), l1 = *reinterpret_cast<const float4 *>(scal + 8 * quad + 4);
      const float4 d0 = *reinterpret_cast<const float4 *>(scal + 32 + 8 * quad), d1 = *reinterpret_cast<const float4 *>(scal + 36 + 8 * quad);
      const float4 g0 = *reinterpret_cast<const float4 *>(scal + 64 + 8 * quad), g1 = *reinterpret_cast<const float4 *>(scal + 68 + 8 * quad);
      lse2[0] = l0.x; lse2[1] = l0.y; lse2[2] = l0.z; lse2[3] = l0.w; lse2[4] = l1.x; lse2[5] = l1.y; lse2[6] = l1.z; lse2[7] = l1.w;
      delta[0] = d0.x; delta[1] = d0.y; delta[2] = d0.z; delta[3] = d0.w; delta[4] = d1.x; delta[5] = d1.y; delta[6] = d1.z; delta[7] = d1.w;
      gw[0] = g0.x; gw[1] = g0.y; gw[2] = g0.z; gw[3] = g0.w; gw[4] = g1.x; gw[5] = g1.y; gw[6] = g1.z; gw[7] = g1.w;
    }
    bf16x8 qt[D / 16], dot[D / 16];
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      qt[dt] = lds_tr_operand<D>(Qr, dt);
      dot[dt] = lds_tr_operand<D>(Dr, dt);
    }
#pragma unroll
    for (int kbk = 0; kbk < KB; ++kbk) {
      bf16x8 pw, ds;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float sv = j < 4 ? s[kbk][0][j & 3] : s[kbk][1][j & 3];
        const float dpv = j < 4 ? dp[kbk][0][j & 3] : dp[kbk][1][j & 3];
        const float p = fast_exp2(__builtin_fmaf(sv, sl2, -lse2[j]));
        pw[j] = (__bf16)(p * gw[j]);
        ds[j] = (__bf16)(p * __builtin_fmaf(gw[j] * scale, dpv, -delta[j] * scale));
      }
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        dv[kbk][dt] = mfma16(dot[dt], pw, dv[kbk][dt]);
        dk[kbk][dt] = mfma16(qt[dt], ds, dk[kbk][dt]);
      }
    }
  }
  if (!wave_on) return;
  // --- store: lane holds dims 16*dt + 4*quad + i of key column n
#pragma unroll
  for (int kbk = 0; kbk < KB; ++kbk) {
    const int key = k0 + 16 * kbk + n;
    if (key >= kend) continue;
    size_t off = ((size_t)key * a.v.Hkv + g) * D + 4 * quad;
    if (MODE == DKV_CMP) off += (size_t)blockIdx.z * a.v.Nc * kstride;
    if (MODE == DKV_SLC) off = (out_row0 + (size_t)(key - kbeg)) * D + 4 * quad;  // partial sums: [row][D]
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      *reinterpret_cast<float4 *>(a.dK + off + 16 * dt) =
          make_float4(dk[kbk][dt][0], dk[kbk][dt][1], dk[kbk][dt][2], dk[kbk][dt][3]);
      *reinterpret_cast<float4 *>(a.dV + off + 16 * dt) =
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
// Inverse of the selection: for every (KV head, selection block) the ascending list of query positions that
// selected it.  Built from a bit matrix (integer OR: order independent), then compacted in order.
// ---------------------------------------------------------------------------------------------------------
__global__ void m_fill_u32(uint32_t *p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void m_sel_bits(const int32_t *__restrict__ idx, const int32_t *__restrict__ perm, int N, int Hkv, int T, int Ns,
                           int words, uint32_t *bits) {
  const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (size_t)N * Hkv * T) return;
  const int pos = (int)(e / ((size_t)Hkv * T)), g = (int)(e / T % Hkv), j = (int)(e % T);
  const int b = idx[((size_t)perm[pos] * Hkv + g) * T + j];
  if (b < 0 || b >= Ns) return;
  atomicOr(&bits[((size_t)g * Ns + b) * words + (pos >> 5)], 1u << (pos & 31));
}

// The same bit matrix built tile by tile in LDS: workgroup (chunk, g) owns `cw` words = 32*cw sorted positions of all
// Ns blocks of KV head g, sets the bits with LDS atomics and writes every word of its tile (so the matrix needs no
// clearing beforehand).  Needs Ns * cw * 4 bytes of LDS.
__global__ __launch_bounds__(256) void m_sel_bits_tile(const int32_t *__restrict__ idx, const int32_t *__restrict__ perm, int N,
                                                       int Hkv, int T, int Ns, int words, int cw, uint32_t *__restrict__ bits) {
  extern __shared__ __align__(16) unsigned char sel_smem[];
  uint32_t *tile = (uint32_t *)sel_smem;  // [Ns][cw]
  const int g = blockIdx.y, w0 = blockIdx.x * cw, p0 = w0 * 32;
  for (int i = threadIdx.x; i < Ns * cw; i += 256) tile[i] = 0u;
  __syncthreads();
  const int npos = min(32 * cw, N - p0);
  for (int e = threadIdx.x; e < npos * T; e += 256) {
    const int pl = e / T, j = e % T;
    const int b = idx[((size_t)perm[p0 + pl] * Hkv + g) * T + j];
    if (b >= 0 && b < Ns) atomicOr(&tile[b * cw + (pl >> 5)], 1u << (pl & 31));
  }
  __syncthreads();
  const int wn = min(cw, words - w0);
  for (int i = threadIdx.x; i < Ns * cw; i += 256) {
    const int b = i / cw, w = i % cw;
    if (w < wn) bits[((size_t)g * Ns + b) * words + w0 + w] = tile[i];
  }
}

__global__ __launch_bounds__(256) void m_sel_count(const uint32_t *__restrict__ bits, int words, uint32_t *counts) {
  __shared__ uint32_t part[4];
  const uint32_t *row = bits + (size_t)blockIdx.x * words;
  uint32_t c = 0;
  for (int i = threadIdx.x; i < words; i += 256) c += __popc(row[i]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) counts[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// single workgroup: from the per-(g, block) selector counts, three exclusive prefix sums over the n keys:
// start (list offsets), chunk_start (work chunks of chunk_len query tokens), part_row_start (rows of partial sums:
// chunks x keys of the block).
__global__ void m_scan_counts(const uint32_t *counts, int n, int Ns, int chunk_len, const int32_t *slc_start,
                              int32_t *start, int32_t *chunk_start, int32_t *part_row_start) {
  __shared__ uint32_t part[3][1024];
  const int tid = threadIdx.x;
  const int per = (n + 1023) / 1024;
  const int b = min(n, tid * per), e = min(n, b + per);
  uint32_t s[3] = {0u, 0u, 0u};
  for (int i = b; i < e; ++i) {
    const uint32_t c = counts[i], nch = (c + chunk_len - 1) / chunk_len;
    const int blk = i % Ns;
    s[0] += c; s[1] += nch; s[2] += nch * (uint32_t)(slc_start[blk + 1] - slc_start[blk]);
  }
  for (int x = 0; x < 3; ++x) part[x][tid] = s[x];
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    uint32_t v[3];
    for (int x = 0; x < 3; ++x) v[x] = tid >= off ? part[x][tid - off] : 0u;
    __syncthreads();
    for (int x = 0; x < 3; ++x) part[x][tid] += v[x];
    __syncthreads();
  }
  uint32_t run[3];
  for (int x = 0; x < 3; ++x) run[x] = part[x][tid] - s[x];
  for (int i = b; i < e; ++i) {
    const uint32_t c = counts[i], nch = (c + chunk_len - 1) / chunk_len;
    const int blk = i % Ns;
    start[i] = (int32_t)run[0]; chunk_start[i] = (int32_t)run[1]; part_row_start[i] = (int32_t)run[2];
    run[0] += c; run[1] += nch; run[2] += nch * (uint32_t)(slc_start[blk + 1] - slc_start[blk]);
  }
  if (tid == 1023) {
    start[n] = (int32_t)part[0][1023]; chunk_start[n] = (int32_t)part[1][1023]; part_row_start[n] = (int32_t)part[2][1023];
  }
}

__global__ __launch_bounds__(256) void m_sel_fill(const uint32_t *__restrict__ bits, int words,
                                                  const int32_t *__restrict__ start, int32_t *list) {
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t base;
  const uint32_t *row = bits + (size_t)blockIdx.x * words;
  if (threadIdx.x == 0) base = (uint32_t)start[blockIdx.x];
  __syncthreads();
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  for (int i0 = 0; i0 < words; i0 += 256) {
    const int i = i0 + threadIdx.x;
    uint32_t w = i < words ? row[i] : 0u;
    const uint32_t c = __popc(w);
    uint32_t incl = c;  // inclusive scan inside the wavefront
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
    if (lane == 63) wsum[wid] = incl;
    __syncthreads();
    uint32_t off = base + incl - c;
    for (int ww = 0; ww < wid; ++ww) off += wsum[ww];
    while (w) {
      const int bit = __ffs(w) - 1;
      list[off++] = i * 32 + bit;
      w &= w - 1;
    }
    __syncthreads();
    if (threadIdx.x == 0) base += wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
  }
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

constexpr int DQ_SLC_WAVES = 4;  // wavefronts per workgroup of the selection dQ kernel (8 tokens at h_s = 8)
constexpr int KB_KEYS_MAX = 2;  // key blocks of 16 per wavefront in the dK/dV kernels (1 at head_dim 128: registers)
// wavefronts per workgroup there (16*KB_KEYS keys each): blocks and windows hold ~130 tokens, an item's pooled keys
// thousands, so the compression branch takes wider workgroups (fewer passes over the query rows)
constexpr int DKV_WAVES = 4, DKV_WAVES_CMP = 8;

template <int D>
int launch_backward(const MfmaView &v, const BwdBuffers &w, const void *q, const void *gates, const void *out_branch,
                    const float *lse, const int32_t *idx, const void *dout, void *dq, void *dk, void *dv, void *dgates,
                    const ssa_blocks *blk, int B, hipStream_t s) {
  const int N = v.N, Hq = v.Hq, Hkv = v.Hkv, row = Hkv * D;
  const size_t NH = (size_t)N * Hq;
  {
    ProfScope ps(PROF_BWD_PRE, s);
    PreArgs a{(const bf16_t *)q, (const bf16_t *)dout, (const bf16_t *)out_branch, (const bf16_t *)gates, lse, v.perm,
              N, Hq, Hkv, v.hs, D, (bf16_t *)dgates, w.lse2s, w.deltas, w.gws, w.Qs, w.dOs};
    m_bwd_pre<<<N, 256, (size_t)Hq * D * sizeof(bf16_t), s>>>(a);
  }
  {
    DqArgs a{v, (const bf16_t *)q, (const bf16_t *)dout, idx, w.lse2s, w.deltas, w.gws, (bf16_t *)dq, w.dQp, nullptr, blk->inv_perm};
    constexpr int CB = 1, NW0 = 4, NW1 = DQ_SLC_WAVES;
    const int tw0 = NW0 * CB * 16 / v.hs, tw1 = NW1 * CB * 16 / v.hs;
    static bool attr_done = false;
    if (!attr_done) {
      (void)hipFuncSetAttribute((const void *)m_bwd_dq<D, CB, 0, NW0>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      (void)hipFuncSetAttribute((const void *)m_bwd_dq<D, CB, 1, NW1>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      attr_done = true;
    }
    {
      ProfScope ps0(PROF_BWD_DQ_CMP, s);
      m_bwd_dq<D, CB, 0, NW0><<<dim3(xcd_grid_size((N + tw0 - 1) / tw0, Hkv)), 64 * NW0, dq_lds_bytes<D>(tw0, v.T, v.Ns), s>>>(a);
    }
    {
      const int rc = slc_order_build(idx, v.perm, N, Hkv, v.T, v.Ns, w.order_ws, s, &a.slc_order);
      if (rc != SSA_OK) return rc;
    }
    {
      ProfScope ps1(PROF_BWD_DQ, s);
      m_bwd_dq<D, CB, 1, NW1><<<dim3(xcd_grid_size((N + tw1 - 1) / tw1, Hkv)), 64 * NW1, dq_lds_bytes<D>(tw1, v.T, v.Ns), s>>>(a);
    }
  }
  constexpr int KB_KEYS = D >= 128 ? 1 : KB_KEYS_MAX;
  constexpr int WG_KEYS = 16 * KB_KEYS * DKV_WAVES, WG_KEYS_CMP = 16 * KB_KEYS * DKV_WAVES_CMP;
  static_assert(WG_KEYS <= SSA_KEY_PAD && WG_KEYS_CMP <= SSA_KEY_PAD, "key tiles may read up to WG_KEYS rows past a block");
  const size_t dkv_lds = (size_t)2 * DkvStage<D>::BYTES;
  static bool dkv_attr = false;
  if (!dkv_attr) {
    (void)hipFuncSetAttribute((const void *)m_bwd_dkv<D, KB_KEYS, DKV_WIN, DKV_WAVES>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    (void)hipFuncSetAttribute((const void *)m_bwd_dkv<D, KB_KEYS, DKV_SLC, DKV_WAVES>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    (void)hipFuncSetAttribute((const void *)m_bwd_dkv<D, KB_KEYS, DKV_CMP, DKV_WAVES_CMP>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    dkv_attr = true;
  }
  DkvArgs base{v, w.Qs, w.dOs, nullptr, nullptr, nullptr, w.sel_start, w.sel_list,
               w.dKs, w.dVs, w.chunk_start, w.part_row_start, w.chunk_len, 1, 1};
  {
    ProfScope ps(PROF_BWD_DKV_WIN, s);
    DkvArgs a = base;
    a.lse2s = w.lse2s + 2 * NH; a.deltas = w.deltas + 2 * NH; a.gws = w.gws + 2 * NH;
    a.tiles_per_block = (blk->win_tok_max + WG_KEYS - 1) / WG_KEYS;
    m_bwd_dkv<D, KB_KEYS, DKV_WIN, DKV_WAVES><<<dim3(blk->Nw * a.tiles_per_block, Hkv), 64 * DKV_WAVES, dkv_lds, s>>>(a);
  }
  {
    ProfScope ps(PROF_BWD_INVERT, s);
    const int words = (N + 31) / 32, keys = Hkv * v.Ns;
    // bit matrix: tiles of up to 32 words per block row held in LDS (64 KB), or global atomics when a KV head has more
    // than 16 384 blocks
    int cw = v.Ns > 0 ? 16384 / v.Ns : 0;
    if (cw > 32) cw = 32;
    if (cw >= 1) {
      m_sel_bits_tile<<<dim3((words + cw - 1) / cw, Hkv), 256, (size_t)v.Ns * cw * 4, s>>>(idx, v.perm, N, Hkv, v.T, v.Ns, words,
                                                                                            cw, w.sel_bits);
    } else {
      m_fill_u32<<<1024, 256, 0, s>>>(w.sel_bits, (size_t)keys * words, 0u);
      const size_t entries = (size_t)N * Hkv * v.T;
      m_sel_bits<<<(unsigned)((entries + 255) / 256), 256, 0, s>>>(idx, v.perm, N, Hkv, v.T, v.Ns, words, w.sel_bits);
    }
    m_sel_count<<<keys, 256, 0, s>>>(w.sel_bits, words, w.sel_counts);
    m_scan_counts<<<1, 1024, 0, s>>>(w.sel_counts, keys, v.Ns, w.chunk_len, v.slc_start, w.sel_start, w.chunk_start,
                                     w.part_row_start);
    m_sel_fill<<<keys, 256, 0, s>>>(w.sel_bits, words, w.sel_start, w.sel_list);
  }
  {
    ProfScope ps(PROF_BWD_DKV_SLC, s);
    DkvArgs a = base;
    a.lse2s = w.lse2s + NH; a.deltas = w.deltas + NH; a.gws = w.gws + NH;
    a.dK = w.pK; a.dV = w.pV;
    a.tiles_per_block = (blk->slc_tok_max + WG_KEYS - 1) / WG_KEYS;
    m_bwd_dkv<D, KB_KEYS, DKV_SLC, DKV_WAVES><<<dim3((w.max_chunks + 7) / 8 * 8 * a.tiles_per_block), 64 * DKV_WAVES, dkv_lds, s>>>(a);
    const size_t items = (size_t)N * Hkv * (D / 4);
    m_slc_reduce<<<(unsigned)((items + 255) / 256), 256, 0, s>>>(blk->tok_slc, v.slc_start, w.chunk_start, w.part_row_start, N,
                                                                 Hkv, v.Ns, D, w.pK, w.pV, w.dKs, w.dVs);
  }
  {
    ProfScope ps(PROF_BWD_DKV_CMP, s);
    DkvArgs a = base;
    a.lse2s = w.lse2s; a.deltas = w.deltas; a.gws = w.gws;
    a.dK = w.dKc; a.dV = w.dVc;
    a.tiles_per_block = (blk->c_max + WG_KEYS_CMP - 1) / WG_KEYS_CMP;
    a.q_splits = w.q_splits;
    m_bwd_dkv<D, KB_KEYS, DKV_CMP, DKV_WAVES_CMP><<<dim3(B * a.tiles_per_block, Hkv, w.q_splits), 64 * DKV_WAVES_CMP, dkv_lds, s>>>(a);
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
