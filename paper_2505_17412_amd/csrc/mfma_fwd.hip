// bf16 MFMA forward kernels of SSA (paper eq. (4)-(6), Algorithm 1, window paragraph) for gfx950.
//
// Compression and window kernels: a workgroup of 4 wavefronts owns 4*CB*16 query rows = consecutive sorted tokens x
// the h_s heads of one KV group; each wavefront keeps CB blocks of 16 query columns and their running softmax state
// (Algorithm 1's m, l, o) in registers.  The selection kernel turns the loops round (per selected block, over the
// tokens that selected it: see the block-centric section below) with the same tile arithmetic.  Scores are produced TRANSPOSED (S^T = K Q^T, keys x queries) so that the
// probabilities land in the lanes exactly as the B operand of the second contraction O^T = V^T P^T needs them.
// Key tiles (K rows and V rows, both row-major) are staged through LDS once per workgroup (see mfma_qc.h); the K
// operand is one 16-byte LDS read, the V^T operand comes from the same row-major V tile through the transposing
// LDS read of gfx950, so no transposed copy of V exists anywhere.
#include "mfma_common.h"
#include "topk_device.h"
#include "mfma_launch.h"
#include "mfma_qc.h"
#include "mfma_bc.h"
#include "profile.h"

#include <mutex>

namespace {

struct FwdArgs {
  MfmaView v;
  const bf16_t *Q;
  bf16_t *Ob;    // [3,N,Hq,D]
  float *lse;    // [3,N,Hq]
  int32_t *idx;  // [N,Hkv,T]
};

// Raw transposed scores of the staged 32-key tile: s[cb][j] = <q column n of block cb, key kb + 8*quad + j>.
template <int D, int CB>
__device__ inline void score_tile(lds_cptr kt, const typename PTile<D>::Lanes &ln, const QRows<D, CB> &q, const bool (&act)[CB],
                                  float (&s)[CB][8]) {
  f32x4 s0[CB], s1[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) s0[cb] = s1[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    const bf16x8 a0 = p_row_operand<D>(kt, ln, 0, ks), a1 = p_row_operand<D>(kt, ln, 1, ks);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      if (act[cb]) {
        s0[cb] = mfma16(a0, q.qop[cb][ks], s0[cb]);
        s1[cb] = mfma16(a1, q.qop[cb][ks], s1[cb]);
      }
  }
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s[cb][i] = s0[cb][i];
      s[cb][4 + i] = s1[cb][i];
    }
}

// One online-softmax step (Algorithm 1, inner loop body) over the staged tile.
//   kt/vt: the staged K and V tiles, ln: the lane offsets of their operands (see PTile);
//   lo/hi: the keys each lane may see (used only when MASK);  on: this lane's column takes part in the tile at all
//   (a token that did not select the current block is off);  act: wave-uniform "some lane of the block is on".
// The reference maximum m of a column is raised lazily: only when some score exceeds it by more than 8 in log2
// units (so every exp2 argument stays below 8 and nothing overflows) does the wavefront take the update path
// with its cross-lane maximum and rescale of o and l; otherwise the tile needs no cross-lane traffic at all.
// The log-sum-exp reported at the end does not depend on which reference was used.
template <int D, int CB, bool MASK>
__device__ inline void fwd_tile(FwdState<D, CB> &st, const QRows<D, CB> &q, lds_cptr kt, lds_cptr vt,
                                const typename PTile<D>::Lanes &ln, int kb,
                                const int (&lo)[CB], const int (&hi)[CB], const bool (&on)[CB], const bool (&act)[CB],
                                float sl2, float slack, const bf16x8 &ones) {
  const int quad = threadIdx.x >> 4 & 3;
  float s[CB][8];
  score_tile<D, CB>(kt, ln, q, act, s);
  bf16x8 pb[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    if (!act[cb]) continue;
    float(&v)[8] = s[cb];
    if (MASK) {
      // lo <= key < hi as one unsigned comparison of (key - lo) against the range length
      const int rel = kb + 8 * quad - lo[cb];
      const unsigned len = (unsigned)(hi[cb] - lo[cb]);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if ((unsigned)(rel + j) >= len) v[j] = -INFINITY;
    }
    float pm = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
    if (!on[cb]) pm = -INFINITY;
    if (__builtin_expect(__any(pm > st.m[cb] + slack), 0)) {  // rare after the first tiles: keep the common path free of copies
      float tmax = fmaxf(pm, __shfl_xor(pm, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float mn = fmaxf(st.m[cb], tmax);
      const float alpha = mn == -INFINITY ? 1.0f : fast_exp2((st.m[cb] - mn) * sl2);
      st.l[cb][0] *= alpha;
      st.m[cb] = mn;
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) st.o[cb][dt] *= alpha;
    }
    // exp2 arguments: finite or -inf; a column that is off (or has seen nothing yet and sees nothing now) gets p = 0
    const float neg = (on[cb] && st.m[cb] != -INFINITY) ? -st.m[cb] * sl2 : -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) pb[cb][j] = (__bf16)fast_exp2(__builtin_fmaf(v[j], sl2, neg));
    // the normaliser on the matrix pipe: an all-ones A operand sums the 32 probabilities of every column, in the
    // same bf16 rounding the numerator uses, and leaves the total in every lane of the column
    st.l[cb] = mfma16(ones, pb[cb], st.l[cb]);
  }
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) {
    const bf16x8 av = p_tr_operand<D>(vt, ln, dt);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      if (act[cb]) st.o[cb][dt] = mfma16(av, pb[cb], st.o[cb][dt]);
  }
}

// Normalise (Algorithm 1: o * exp(m - l)), store the branch output and its log-sum-exp; lse2[cb] in log2 units.
template <int D, int CB>
__device__ inline void finish(const FwdArgs &a, FwdState<D, CB> &st, int branch, const QRows<D, CB> &q, float (&lse2)[CB]) {
  const int quad = threadIdx.x >> 4 & 3;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const float l = st.l[cb][0];
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    lse2[cb] = l > 0.f ? st.m[cb] * a.v.sl2 + __log2f(l) : -INFINITY;
    if (q.valid[cb]) {
      bf16_t *o = a.Ob + (((size_t)branch * a.v.N + q.tok[cb]) * a.v.Hq + q.h[cb]) * D;
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        bf16x4 w;
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (__bf16)(st.o[cb][dt][i] * inv);
        *reinterpret_cast<bf16x4 *>(o + acc_dim(dt, quad)) = w;
      }
      if (quad == 0) a.lse[((size_t)branch * a.v.N + q.tok[cb]) * a.v.Hq + q.h[cb]] = lse2[cb] * LN2;
    }
  }
}

constexpr float SCORE_FIX = 134217728.0f;  // 2^27: a row's scores sum to h_s <= 16 < 2^5

// LDS plan of the compression kernel (bytes): two tile stages | 8 ints | scores [TW][s_max] | top-k marks [4][words] |
// lse per query row [4 waves][CB <= 4][16]
template <int D>
__host__ __device__ inline size_t cmp_lds_bytes(int tw, int s_max) {
  return (size_t)2 * StageLayout<D, 2>::ELEMS * sizeof(bf16_t) + 32 + ((size_t)tw * s_max + 4 * ((s_max + 31) / 32) + 4 * 4 * 16) * 4;
}

// Compression branch (eq. (4) first term over the mean-pooled keys of eq. (5)), then the selection scores of
// eq. (6) accumulated per selection block in LDS as fixed-point integers (integer adds commute, so the result
// does not depend on scheduling), then the top-k.
template <int D, int CB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D <= 64 ? 4 : 2))) void m_cmp_fwd(FwdArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  using L = StageLayout<D, 2>;
  bf16_t *stage0 = (bf16_t *)smem;
  int *ints = (int *)(stage0 + 2 * L::ELEMS);
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int hs = a.v.hs, s_max = a.v.s_max, TW = 4 * CB * 16 / hs;
  const TileMap tm = xcd_tile_map((a.v.N + TW - 1) / TW, a.v.Hkv);
  if (!tm.valid) return;
  const int g = tm.g, wg_pos0 = tm.tile * TW;
  uint32_t *S = (uint32_t *)(ints + 8);
  uint32_t *sel_base = S + (size_t)TW * s_max;
  uint32_t *sel = sel_base + (size_t)wid * ((s_max + 31) >> 5);
  QRows<D, CB> q;
  load_rows<D, CB>(a.Q, a.v, wg_pos0, g, q);
  int lo[CB], hi[CB], s0[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int item = q.valid[cb] ? a.v.tok_item[q.pos[cb]] : 0;
    lo[cb] = q.valid[cb] ? a.v.cmp_batch[item] : 0;
    hi[cb] = q.valid[cb] ? a.v.cmp_batch[item + 1] : 0;
    s0[cb] = q.valid[cb] ? a.v.slc_batch[item] : 0;
  }
  int rs, re;
  bool uniform;
  wg_range<CB>(ints, lo, hi, q.valid, rs, re, uniform);
  if (threadIdx.x == 0) { ints[4] = rs; ints[5] = re; }
  __syncthreads();
  const int nr = re > rs ? 1 : 0;
  bool act[CB], on[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) { act[cb] = true; on[cb] = q.valid[cb]; }
  const float slack = 8.0f / a.v.sl2;
  TileSrc<2> src{{a.v.Kc + (size_t)g * D, a.v.Vc + (size_t)g * D}, (uint32_t)(a.v.Hkv * D)};
  FwdState<D, CB> st;
  init_state(st);
  const bf16x8 ones = ones_operand();
  const float sl2 = a.v.sl2;
  const typename PTile<D>::Lanes ln = PTile<D>::lanes();
  run_pipeline<D, 2>(
      src, stage0, ints + 4, ints + 5, nr, [](int) {},
      [&](const bf16_t *stg, int kb, int) {
        if (uniform && kb >= rs && kb + 32 <= re)
          fwd_tile<D, CB, false>(st, q, (lds_cptr)L::row_tile((bf16_t *)stg, 0), (lds_cptr)L::row_tile((bf16_t *)stg, 1), ln, kb, lo, hi, on, act, sl2, slack, ones);
        else
          fwd_tile<D, CB, true>(st, q, (lds_cptr)L::row_tile((bf16_t *)stg, 0), (lds_cptr)L::row_tile((bf16_t *)stg, 1), ln, kb, lo, hi, on, act, sl2, slack, ones);
      });
  float lse2[CB];
  finish<D, CB>(a, st, 0, q, lse2);

  // ---- selection scores, eq. (6): second walk over the pooled keys with the normaliser known
  for (int i = threadIdx.x; i < TW * s_max; i += 256) S[i] = 0u;
  TileSrc<1> ksrc{{a.v.Kc + (size_t)g * D}, (uint32_t)(a.v.Hkv * D)};
  if (hs >= 4) {
    // Scores NOT transposed here (S = Q K^T: query rows x keys), so that a lane holds four heads of ONE token for
    // one key: the sum over the group's heads (eq. (6), inner sum) is three in-lane adds plus at most two lane
    // exchanges, and one integer LDS atomic per (token, key) adds it onto the key's selection block (outer sum).
    float *lse_l = (float *)(sel_base + 4 * ((s_max + 31) >> 5));  // [4 waves][CB][16] lse2 per query row
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      if (quad == 0) lse_l[(wid * CB + cb) * 16 + n] = lse2[cb];
    __syncthreads();
    float l4[CB][4];
    int klo[CB], khi[CB], ks0[CB], kslot[CB];
    bool owner[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
      for (int i = 0; i < 4; ++i) l4[cb][i] = lse_l[(wid * CB + cb) * 16 + 4 * quad + i];
      kslot[cb] = (wid * CB + cb) * (16 / hs) + (4 * quad) / hs;  // the token of this lane's four rows
      const int pos = wg_pos0 + kslot[cb];
      const bool ok = pos < a.v.N;
      const int item = ok ? a.v.tok_item[pos] : 0;
      klo[cb] = ok ? a.v.cmp_batch[item] : 0;
      khi[cb] = ok ? a.v.cmp_batch[item + 1] : 0;
      ks0[cb] = ok ? a.v.slc_batch[item] : 0;
      owner[cb] = (4 * quad) % hs == 0;
    }
    // two consecutive 32-key tiles per step: half the barriers and staging rounds of a walk that has little work per key
    TileSrc<2> ksrc2{{a.v.Kc + (size_t)g * D, a.v.Kc + (size_t)g * D + (size_t)32 * a.v.Hkv * D}, (uint32_t)(a.v.Hkv * D)};
    run_pipeline<D, 2, 256, 2, 64>(
        ksrc2, stage0, ints + 4, ints + 5, nr, [](int) {},
        [&](const bf16_t *stg2, int kb2, int) {
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const bf16_t *stg = L::row_tile((bf16_t *)stg2, half);
            const int kb = kb2 + 32 * half;
            // the selection block of this lane's key in either sub-tile, requested before the matrix instructions
            int sblk[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) sblk[sub] = a.v.cmp_slc[min(tile_key_row(kb, sub), a.v.Nc - 1)];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
              f32x4 c[CB];
#pragma unroll
              for (int cb = 0; cb < CB; ++cb) c[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
              for (int ks = 0; ks < D / 32; ++ks) {
                const bf16x8 kop = p_row_operand<D>((lds_cptr)stg, ln, sub, ks);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) c[cb] = mfma16(q.qop[cb][ks], kop, c[cb]);
              }
              const int key = tile_key_row(kb, sub);  // column n of sub-tile `sub` sits in row slot 16*sub + n
#pragma unroll
              for (int cb = 0; cb < CB; ++cb) {
                float t = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) t += fast_exp2(__builtin_fmaf(c[cb][i], sl2, -l4[cb][i]));
                if (hs >= 8) t += __shfl_xor(t, 16);
                if (hs >= 16) t += __shfl_xor(t, 32);
                if (owner[cb] && key >= klo[cb] && key < khi[cb])
                  atomicAdd(&S[(size_t)kslot[cb] * s_max + sblk[sub] - ks0[cb]], (uint32_t)(t * SCORE_FIX));
              }
            }
          }
        });
  } else {
    __syncthreads();
    run_pipeline<D, 1>(
        ksrc, stage0, ints + 4, ints + 5, nr, [](int) {},
        [&](const bf16_t *stg, int kb, int) {
          float s[CB][8];
          score_tile<D, CB>((lds_cptr)stg, ln, q, act, s);
          const int hl = n % hs;
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) {
            float p[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              p[j] = fast_exp2(__builtin_fmaf(s[cb][j], sl2, -lse2[cb]));
              p[j] = group_sum(p[j], hs);  // sum over the group's heads (eq. (6), inner sum)
            }
            // every lane of a head group now holds the same 8 sums; lane hl adds the sums of keys j = hl (mod hs)
            // onto their selection blocks (eq. (6), outer sum over the child blocks)
            uint32_t *Srow = S + (size_t)q.slot[cb] * s_max;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const int key = kb + 8 * quad + j;
              if (q.valid[cb] && (j % hs) == hl && key >= lo[cb] && key < hi[cb])
                atomicAdd(&Srow[a.v.cmp_slc[key] - s0[cb]], (uint32_t)(p[j] * SCORE_FIX));
            }
          }
        });
  }
  // ---- top-k: each wavefront serves its own token slots, one after the other
  const int spw = CB * 16 / hs;  // token slots per wavefront
  for (int tl = 0; tl < spw; ++tl) {
    const int slot = wid * spw + tl, pos = wg_pos0 + slot;
    if (pos >= a.v.N) break;
    const int tok = a.v.perm[pos], it = a.v.tok_item[pos];
    const int b0 = a.v.slc_batch[it], nb = a.v.slc_batch[it + 1] - b0;
    int32_t *row = a.idx + ((size_t)tok * a.v.Hkv + g) * a.v.T;
    if (s_max <= 512) topk_wave_bits<8>(S + (size_t)slot * s_max, nb, a.v.T, b0, row);
    else if (s_max <= 1024) topk_wave_bits<16>(S + (size_t)slot * s_max, nb, a.v.T, b0, row);
    else topk_wave_u32(S + (size_t)slot * s_max, nb, a.v.T, b0, row, sel);
  }
}

// Window branch: keys are the tokens of the query's own window.
template <int D, int CB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D <= 64 ? 4 : 2))) void m_win_fwd(FwdArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  using L = StageLayout<D, 2>;
  bf16_t *stage0 = (bf16_t *)smem;
  int *ints = (int *)(stage0 + 2 * L::ELEMS);
  const int hs = a.v.hs, TW = 4 * CB * 16 / hs;
  const TileMap tm = xcd_tile_map((a.v.N + TW - 1) / TW, a.v.Hkv);
  if (!tm.valid) return;
  const int g = tm.g, wg_pos0 = tm.tile * TW;
  QRows<D, CB> q;
  load_rows<D, CB>(a.Q, a.v, wg_pos0, g, q);
  int lo[CB], hi[CB];
  bool act[CB], on[CB];
  const float slack = 8.0f / a.v.sl2;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int w = q.valid[cb] ? a.v.tok_win[q.pos[cb]] : 0;
    lo[cb] = q.valid[cb] ? a.v.win_start[w] : 0;
    hi[cb] = q.valid[cb] ? a.v.win_start[w + 1] : 0;
    act[cb] = true;
    on[cb] = q.valid[cb];
  }
  int rs, re;
  bool uniform;
  wg_range<CB>(ints, lo, hi, q.valid, rs, re, uniform);
  if (threadIdx.x == 0) { ints[4] = rs; ints[5] = re; }
  __syncthreads();
  TileSrc<2> src{{a.v.Ks + (size_t)g * D, a.v.Vs + (size_t)g * D}, (uint32_t)(a.v.Hkv * D)};
  FwdState<D, CB> st;
  init_state(st);
  const bf16x8 ones = ones_operand();
  const float sl2 = a.v.sl2;
  const typename PTile<D>::Lanes ln = PTile<D>::lanes();
  run_pipeline<D, 2>(
      src, stage0, ints + 4, ints + 5, re > rs ? 1 : 0, [](int) {},
      [&](const bf16_t *stg, int kb, int) {
        if (uniform && kb >= rs && kb + 32 <= re)
          fwd_tile<D, CB, false>(st, q, (lds_cptr)L::row_tile((bf16_t *)stg, 0), (lds_cptr)L::row_tile((bf16_t *)stg, 1), ln, kb, lo, hi, on, act, sl2, slack, ones);
        else
          fwd_tile<D, CB, true>(st, q, (lds_cptr)L::row_tile((bf16_t *)stg, 0), (lds_cptr)L::row_tile((bf16_t *)stg, 1), ln, kb, lo, hi, on, act, sl2, slack, ones);
      });
  float lse2[CB];
  finish<D, CB>(a, st, 2, q, lse2);
}

constexpr int FWD_CB = 1;
constexpr int CMP_CB = 1;     // 16-column blocks per wavefront of the compression kernel

template <int D>
int launch_forward(FwdArgs a, const bf16_t *gates, bf16_t *out, const SelIndex &sel, const SlcPartials &part, hipStream_t s) {
  const int tw = 4 * FWD_CB * 16 / a.v.hs, tw_cmp = 4 * CMP_CB * 16 / a.v.hs;
  const dim3 grid(xcd_grid_size((a.v.N + tw - 1) / tw, a.v.Hkv));
  const size_t lds_cmp = cmp_lds_bytes<D>(tw_cmp, a.v.s_max);
  const size_t lds_win = (size_t)2 * StageLayout<D, 2>::ELEMS * sizeof(bf16_t) + 32;
  static std::once_flag attr_once;  // raise the dynamic LDS limit once per process for this instantiation
  std::call_once(attr_once, [] {
    (void)hipFuncSetAttribute((const void *)m_cmp_fwd<D, CMP_CB>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  });
  {
    ProfScope ps(PROF_CMP_FWD, s);
    m_cmp_fwd<D, CMP_CB><<<dim3(xcd_grid_size((a.v.N + tw_cmp - 1) / tw_cmp, a.v.Hkv)), 256, lds_cmp, s>>>(a);
  }
  {
    ProfScope ps(PROF_FWD_INVERT, s);
    const int rc = sel_index_build(a.idx, a.v.perm, a.v.slc_start, a.v.N, a.v.Hkv, a.v.T, a.v.Ns, sel, false, s);
    if (rc != SSA_OK) return rc;
  }
  {
    ProfScope ps(PROF_SLC_FWD, s);
    const int rc = slc_forward_kernel(a.v, D, a.Q, a.idx, sel, part, s);
    if (rc != SSA_OK) return rc;
  }
  {
    ProfScope ps(PROF_WIN_FWD, s);
    m_win_fwd<D, FWD_CB><<<grid, 256, lds_win, s>>>(a);
  }
  {
    ProfScope ps(PROF_COMBINE, s);
    const int rc = slc_merge_kernel(a.v, D, part, a.idx, gates, a.Ob, a.lse, out, s);
    if (rc != SSA_OK) return rc;
  }
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

}  // namespace

// Largest dynamic LDS request of the forward kernels for this problem (bytes).
size_t mfma_fwd_lds_bytes(int D, int hs, int s_max) {
  const int tw = 4 * CMP_CB * 16 / hs;
  switch (D) {
    case 32: return cmp_lds_bytes<32>(tw, s_max);
    case 64: return cmp_lds_bytes<64>(tw, s_max);
    default: return cmp_lds_bytes<128>(tw, s_max);
  }
}

int mfma_forward_kernels(const MfmaView &v, int D, const void *q, const void *gates, void *out, float *lse,
                         int32_t *idx, void *out_branch, const SelIndex &sel, const SlcPartials &part, hipStream_t s) {
  FwdArgs a{v, (const bf16_t *)q, (bf16_t *)out_branch, lse, idx};
  switch (D) {
    case 32: return launch_forward<32>(a, (const bf16_t *)gates, (bf16_t *)out, sel, part, s);
    case 64: return launch_forward<64>(a, (const bf16_t *)gates, (bf16_t *)out, sel, part, s);
    case 128: return launch_forward<128>(a, (const bf16_t *)gates, (bf16_t *)out, sel, part, s);
    default: return SSA_ERR_UNSUPPORTED;
  }
}
