// Selection branch of SSA on bf16 MFMA for gfx950, block-centric: Algorithm 1 with its two loops exchanged, forward and
// dQ, and the kernels that merge the per-block partial results (the forward one also forms the gated sum of eq. (4)).
// A translation unit of its own: these kernels have no barrier in their inner loops and long straight-line tile code,
// and are compiled with an instruction scheduler setting of their own (see build.py).
#include "mfma_common.h"
#include "mfma_launch.h"
#include "mfma_qc.h"
#include "mfma_bc.h"

#include <mutex>

namespace {

// ---------------------------------------------------------------------------------------------------------
// Selection branch, block-centric (Algorithm 1 with the loops exchanged): the outer loop runs over the selected blocks,
// the inner one over the query tokens that selected the block.  A workgroup takes one (KV head, selection block) and a
// chunk of up to BC_CHUNK tokens of that block's selector list, puts the block's K and V rows into LDS ONCE (up to KSEG
// keys; longer blocks in several segments) and lets every wavefront run, on its own and without any barrier, through
// groups of CB*16/h_s tokens: all CB*16 query columns of a matrix tile then take part in every key tile (nothing is
// computed for a token that did not select the block), the K and V^T operands read from LDS feed CB column blocks,
// and no wavefront waits for another.  The price is one partial result per (token, KV head, selected block): the
// unnormalised output in bf16 with its running maximum and sum (Algorithm 1's o, m, l for that block alone), merged per
// token afterwards (m_slc_merge).  A wavefront that meets a block longer than KSEG picks its own partial up again for
// the next segment.
// ---------------------------------------------------------------------------------------------------------
struct BcFwdArgs {
  MfmaView v;
  const bf16_t *Q;
  const int32_t *idx;  // [N,Hkv,T]
  const int32_t *sel_start, *sel_list, *chunk_start, *chunk_order;
  bf16_t *po;  // [N][Hkv][T][hs][D]
  float *pml;  // [N][Hkv][T][hs][2]
};

// LDS plan (bytes): K tiles | V tiles (KSEG/32 tiles each, PTile layout) | token ids [BC_CHUNK] | ranks [BC_CHUNK]
template <int D, int KSEG>
constexpr size_t bc_lds_bytes() { return (size_t)2 * (KSEG / 32) * PTile<D, false>::BYTES + (size_t)2 * BC_CHUNK * sizeof(int); }

// Query operands and partial-row index of one wavefront step: column n stands for chunk entry step*(16/h_s) + n/h_s,
// head n % h_s of the KV group.
template <int D>
struct BcRows {
  bf16x8 qop[D / 32];
  uint32_t prow;  // ((tok*Hkv + g)*T + rank)*hs + head: row of the partial arrays (below 2^32: N*Hq*T is)
  bool valid;
};

template <int D>
__device__ inline void bc_load_rows(const BcFwdArgs &a, const int *tl, const int *sl, int step, int cnt, int g, BcRows<D> &r) {
  const int n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
  const int hs = a.v.hs, hl = n % hs;
  const int e = step * (16 / hs) + n / hs;
  r.valid = e < cnt;
  const int tok = r.valid ? tl[e] : 0, rank = r.valid ? sl[e] : 0;
  const bf16_t *src = a.Q + ((size_t)tok * a.v.Hq + g * hs + hl) * D + 8 * quad;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) r.qop[ks] = r.valid ? ld8(src + 32 * ks) : zero8();
  r.prow = (uint32_t)((((size_t)tok * a.v.Hkv + g) * a.v.T + rank) * hs + hl);
}

// One online-softmax step (Algorithm 1, inner loop body) of 16 query columns over one 32-key LDS tile.  kt, vt: the K
// and V tile, ln: the lane offsets of their operands (see PTile).  MASK: keys from index nk on (counted from the segment start;
// this tile starts at key0) do not exist.  Lazy reference maximum as in fwd_tile.
template <int D, bool MASK>
__device__ inline void bc_fwd_tile(FwdState<D, 1> &st, const bf16x8 (&qop)[D / 32], lds_cptr kt, lds_cptr vt,
                                   const typename PTile<D, false>::Lanes &ln, int key0, int nk, float sl2, float slack,
                                   const bf16x8 &ones) {
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    s0 = mfma16(p_row_operand<D, false>(kt, ln, 0, ks), qop[ks], s0);
    s1 = mfma16(p_row_operand<D, false>(kt, ln, 1, ks), qop[ks], s1);
  }
  float v[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
  if (MASK) {
    const int first = key0 + 8 * (int)(threadIdx.x >> 4 & 3);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (first + j >= nk) v[j] = -INFINITY;
  }
  const float pm = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
  if (__builtin_expect(__any(pm > st.m[0] + slack), 0)) {
    float tmax = fmaxf(pm, __shfl_xor(pm, 16));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float mn = fmaxf(st.m[0], tmax);
    const float alpha = mn == -INFINITY ? 1.0f : fast_exp2((st.m[0] - mn) * sl2);
    st.l[0][0] *= alpha;
    st.m[0] = mn;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) st.o[0][dt] *= alpha;
  }
  const float neg = st.m[0] != -INFINITY ? -st.m[0] * sl2 : -INFINITY;
  bf16x8 pb;
#pragma unroll
  for (int j = 0; j < 8; ++j) pb[j] = (__bf16)fast_exp2(__builtin_fmaf(v[j], sl2, neg));
  st.l[0] = mfma16(ones, pb, st.l[0]);
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) st.o[0][dt] = mfma16(p_tr_operand<D, false>(vt, ln, dt), pb, st.o[0][dt]);
}

template <int D, int NW, int KSEG>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(D <= 64 ? 4 : 2))) void m_slc_fwd_bc(BcFwdArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  using P = PTile<D, false>;
  constexpr int MAXT = KSEG / 32;
  unsigned char *Kt = smem, *Vt = Kt + MAXT * P::BYTES;
  int *tl = (int *)(Vt + MAXT * P::BYTES), *sl = tl + BC_CHUNK;
  const int wid = threadIdx.x >> 6, quad = threadIdx.x >> 4 & 3;
  const int hs = a.v.hs, Hkv = a.v.Hkv, T = a.v.T, Ns = a.v.Ns;
  const int wi = bc_chunk_of_workgroup(a.chunk_start[Hkv * Ns]);
  int key, chunk;
  if (wi < 0 || !bc_find_chunk(a.chunk_start, Hkv * Ns, a.chunk_order[wi], key, chunk)) return;
  const int g = key / Ns, blk = key % Ns;
  const int kbeg = a.v.slc_start[blk], kend = a.v.slc_start[blk + 1];
  const int qbeg = a.sel_start[key] + chunk * BC_CHUNK, cnt = min(a.sel_start[key + 1] - qbeg, BC_CHUNK);
  // the chunk's tokens (caller indices) and the rank of this block in each token's row of I
  for (int i = threadIdx.x; i < cnt; i += 64 * NW) {
    const int tok = a.v.perm[a.sel_list[qbeg + i]];
    const int32_t *row = a.idx + ((size_t)tok * Hkv + g) * T;
    int j = 0;
    while (j < T - 1 && row[j] != blk) ++j;
    tl[i] = tok;
    sl[i] = j;
  }
  const int tpw = 16 / hs;  // tokens per wavefront step
  const int n_it = (cnt + tpw - 1) / tpw;
  const uint32_t kstride = (uint32_t)(Hkv * D);
  const float sl2 = a.v.sl2, slack = 8.0f / sl2;
  const bf16x8 ones = ones_operand();
  const typename P::Lanes ln = P::lanes();
  const lds_cptr kl = (lds_cptr)Kt, vl = (lds_cptr)Vt;
  __syncthreads();
  BcRows<D> cur;
  if (wid < n_it) bc_load_rows<D>(a, tl, sl, wid, cnt, g, cur);  // in flight while the block is staged
  for (int k0 = kbeg; k0 < kend; k0 += KSEG) {
    const int nk = min(KSEG, kend - k0), nfull = nk >> 5;
    if (k0 > kbeg) {
      __syncthreads();  // every wavefront is done with the previous segment
      if (wid < n_it) bc_load_rows<D>(a, tl, sl, wid, cnt, g, cur);
    }
    p_stage2<D, false, 64 * NW>(a.v.Ks + (size_t)g * D, a.v.Vs + (size_t)g * D, kstride, k0, (nk + 31) >> 5, Kt, Vt);
    __syncthreads();
    for (int it = wid; it < n_it; it += NW) {
      BcRows<D> nxt;  // the next step's operands are requested before this step's arithmetic
      if (it + NW < n_it) bc_load_rows<D>(a, tl, sl, it + NW, cnt, g, nxt);
      FwdState<D, 1> st;
      init_state(st);
      if (k0 > kbeg && cur.valid) {  // pick the partial of the earlier segments up again
        const float2 ml = *reinterpret_cast<const float2 *>(a.pml + (size_t)cur.prow * 2);
        st.m[0] = ml.x;
        st.l[0][0] = ml.y;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
          const bf16x4 x = *reinterpret_cast<const bf16x4 *>(a.po + (size_t)cur.prow * D + acc_dim(dt, quad));
#pragma unroll
          for (int i = 0; i < 4; ++i) st.o[0][dt][i] = (float)x[i];
        }
      }
#pragma unroll
      for (int t = 0; t < MAXT; ++t)
        if (t < nfull) bc_fwd_tile<D, false>(st, cur.qop, kl + t * P::BYTES, vl + t * P::BYTES, ln, 32 * t, nk, sl2, slack, ones);
      if (nk & 31)
        bc_fwd_tile<D, true>(st, cur.qop, kl + nfull * P::BYTES, vl + nfull * P::BYTES, ln, 32 * nfull, nk, sl2, slack, ones);
      // (a column past the end of the chunk points at row 0 of the partial arrays and is not stored)
      store_partial_row<D>(a.po + (size_t)cur.prow * D, st.o[0], cur.valid);
      if (cur.valid && quad == 0) *reinterpret_cast<float2 *>(a.pml + (size_t)cur.prow * 2) = make_float2(st.m[0], st.l[0][0]);
      cur = nxt;
    }
  }
}

// Merge of the per-block partials of the selection branch (the online-softmax recurrence of Algorithm 1 applied across
// blocks instead of key tiles), and the gate-weighted sum of eq. (4) in the same pass: one thread per (token, query
// head, 8 output dims).  Writes out_branch[1], lse[1] and out.
struct MergeArgs {
  const bf16_t *po;
  const float *pml;
  const int32_t *idx;
  const bf16_t *gates;
  bf16_t *Ob;  // [3,N,Hq,D]: branches 0 and 2 are read, 1 is written
  float *lse;  // [3,N,Hq]
  bf16_t *out;
  int N, Hq, Hkv, hs, T, D;
  float sl2;
};

__global__ __launch_bounds__(256) void m_slc_merge(MergeArgs a) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per_row = a.D / 8;
  if (i >= (size_t)a.N * a.Hq * per_row) return;
  const int c8 = (int)(i % per_row), h = (int)(i / per_row % a.Hq), tok = (int)(i / ((size_t)per_row * a.Hq));
  const int g = h / a.hs, hl = h % a.hs;
  const size_t slot0 = ((size_t)tok * a.Hkv + g) * a.T;
  const int32_t *row = a.idx + slot0;
  int nv = 0;  // rows are ascending with the -1 padding at the end
  for (int j = 0; j < a.T; ++j) nv += row[j] >= 0 ? 1 : 0;
  float M = -INFINITY;
  for (int j = 0; j < nv; ++j) M = fmaxf(M, a.pml[((slot0 + j) * a.hs + hl) * 2]);
  float L = 0.f, acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int j = 0; j < nv; ++j) {
    const size_t r = (slot0 + j) * a.hs + hl;
    const float2 ml = *reinterpret_cast<const float2 *>(a.pml + r * 2);
    const bf16x8 x = ld8(a.po + r * a.D + 8 * c8);
    const float wj = ml.x == -INFINITY ? 0.f : fast_exp2((ml.x - M) * a.sl2);
    L += wj * ml.y;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += wj * (float)x[e];
  }
  const float inv = L > 0.f ? 1.0f / L : 0.f;
  const size_t th = (size_t)tok * a.Hq + h, NH = (size_t)a.N * a.Hq;
  const size_t off = th * a.D + 8 * c8;
  bf16x8 os;
#pragma unroll
  for (int e = 0; e < 8; ++e) os[e] = (__bf16)(acc[e] * inv);
  *reinterpret_cast<bf16x8 *>(a.Ob + NH * a.D + off) = os;
  if (c8 == 0) a.lse[NH + th] = L > 0.f ? (M * a.sl2 + __log2f(L)) * LN2 : -INFINITY;
  const float w0 = bf16_to_f32(a.gates[th * 3]), w1 = bf16_to_f32(a.gates[th * 3 + 1]), w2 = bf16_to_f32(a.gates[th * 3 + 2]);
  const bf16x8 x0 = ld8(a.Ob + off), x2 = ld8(a.Ob + 2 * NH * a.D + off);
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)(w0 * (float)x0[e] + w1 * (float)os[e] + w2 * (float)x2[e]);
  *reinterpret_cast<bf16x8 *>(a.out + off) = o;
}

// ---------------------------------------------------------------------------------------------------------
// dQ of the selection branch, block-centric: the same exchange of loops as the forward kernel m_slc_fwd_bc.  A workgroup
// holds one selection block's K and V rows in LDS and runs through a chunk of the tokens that selected it; every
// wavefront takes 16/h_s tokens per step on its own (query and dO rows in registers, no barrier, no column that did
// not select the block).  One bf16 partial dQ per (token, KV head, selected block) goes to memory; m_dq_merge adds them
// in rank order onto the fp32 compression + window part.
// ---------------------------------------------------------------------------------------------------------
struct BcDqArgs {
  MfmaView v;
  const bf16_t *Qs, *dOs;             // [N(pos)][Hq][D] sorted copies: Q, and the selection gate times dO
  const float *lse2s, *deltas;        // selection branch: [N(pos)][Hq]
  const int32_t *idx;                 // [N,Hkv,T]
  const int32_t *sel_start, *sel_list, *chunk_start, *chunk_order;
  bf16_t *pdq;                        // [N(pos)][Hkv][T][hs][D]
};

template <int D>
struct BcDqRows {
  bf16x8 qop[D / 32], dop[D / 32];
  float lse2, nd;   // lse in log2 units; -delta (delta = gate * <dO, O>)
  uint32_t prow;         // ((pos*Hkv + g)*T + rank)*hs + head
  bool valid;
};

template <int D>
__device__ inline void bc_dq_load_rows(const BcDqArgs &a, const int *tl, const int *sl, int step, int cnt, int g, BcDqRows<D> &r) {
  const int n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
  const int hs = a.v.hs, hl = n % hs;
  const int e = step * (16 / hs) + n / hs;
  r.valid = e < cnt;
  const int pos = r.valid ? tl[e] : 0, rank = r.valid ? sl[e] : 0;
  const size_t th = (size_t)pos * a.v.Hq + g * hs + hl;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    r.qop[ks] = r.valid ? ld8(a.Qs + th * D + 8 * quad + 32 * ks) : zero8();
    r.dop[ks] = r.valid ? ld8(a.dOs + th * D + 8 * quad + 32 * ks) : zero8();
  }
  r.lse2 = r.valid ? a.lse2s[th] : INFINITY;  // a missing column gets P = exp2(-inf) = 0
  r.nd = -a.deltas[th];
  r.prow = (uint32_t)((((size_t)pos * a.v.Hkv + g) * a.v.T + rank) * hs + hl);
}

// One 32-key LDS tile: transposed scores (K rows) and dP (V rows, against gate * dO; the accumulators start from
// -delta of their column, so the matrix instruction leaves dP - delta), dS^T = P (dP - delta), then dQ^T += K^T dS^T
// with K^T read from the same K tile through the transposing LDS load.  The softmax scale of dS is applied by the merge
// kernel, once per output element.
template <int D, bool MASK>
__device__ inline void bc_dq_tile(f32x4 (&acc)[D / 16], const BcDqRows<D> &r, lds_cptr kt, lds_cptr vt,
                                  const typename PTile<D, false>::Lanes &ln, int key0, int nk, float sl2) {
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0, p0 = {r.nd, r.nd, r.nd, r.nd}, p1 = p0;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    s0 = mfma16(p_row_operand<D, false>(kt, ln, 0, ks), r.qop[ks], s0);
    s1 = mfma16(p_row_operand<D, false>(kt, ln, 1, ks), r.qop[ks], s1);
    p0 = mfma16(p_row_operand<D, false>(vt, ln, 0, ks), r.dop[ks], p0);
    p1 = mfma16(p_row_operand<D, false>(vt, ln, 1, ks), r.dop[ks], p1);
  }
  bf16x8 ds;
  const int first = key0 + 8 * (int)(threadIdx.x >> 4 & 3);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float sv = j < 4 ? s0[j & 3] : s1[j & 3], dp = j < 4 ? p0[j & 3] : p1[j & 3];
    float p = fast_exp2(__builtin_fmaf(sv, sl2, -r.lse2));
    if (MASK && first + j >= nk) p = 0.f;
    ds[j] = (__bf16)(p * dp);  // dp = gate * dP - delta: the dO rows are gate * dO
  }
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) acc[dt] = mfma16(p_tr_operand<D, false>(kt, ln, dt), ds, acc[dt]);
}

template <int D, int KSEG>
constexpr size_t bc_dq_lds_bytes() { return (size_t)2 * (KSEG / 32) * PTile<D, false>::BYTES + (size_t)2 * BC_CHUNK * sizeof(int); }

template <int D, int NW, int KSEG>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(D <= 64 ? 4 : 2))) void m_bwd_dq_bc(BcDqArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  using P = PTile<D, false>;
  constexpr int MAXT = KSEG / 32;
  unsigned char *Kt = smem, *Vt = Kt + MAXT * P::BYTES;
  int *tl = (int *)(Vt + MAXT * P::BYTES), *sl = tl + BC_CHUNK;
  const int wid = threadIdx.x >> 6, quad = threadIdx.x >> 4 & 3;
  const int hs = a.v.hs, Hkv = a.v.Hkv, T = a.v.T, Ns = a.v.Ns;
  const int wi = bc_chunk_of_workgroup(a.chunk_start[Hkv * Ns]);
  int key, chunk;
  if (wi < 0 || !bc_find_chunk(a.chunk_start, Hkv * Ns, a.chunk_order[wi], key, chunk)) return;
  const int g = key / Ns, blk = key % Ns;
  const int kbeg = a.v.slc_start[blk], kend = a.v.slc_start[blk + 1];
  const int qbeg = a.sel_start[key] + chunk * BC_CHUNK, cnt = min(a.sel_start[key + 1] - qbeg, BC_CHUNK);
  // the chunk's tokens (sorted positions) and the rank of this block in each token's row of I
  for (int i = threadIdx.x; i < cnt; i += 64 * NW) {
    const int pos = a.sel_list[qbeg + i];
    const int32_t *row = a.idx + ((size_t)a.v.perm[pos] * Hkv + g) * T;
    int j = 0;
    while (j < T - 1 && row[j] != blk) ++j;
    tl[i] = pos;
    sl[i] = j;
  }
  const int tpw = 16 / hs;
  const int n_it = (cnt + tpw - 1) / tpw;
  const uint32_t kstride = (uint32_t)(Hkv * D);
  const float sl2 = a.v.sl2;
  const typename P::Lanes ln = P::lanes();
  const lds_cptr kt = (lds_cptr)Kt, vt = (lds_cptr)Vt;
  __syncthreads();
  BcDqRows<D> cur;
  if (wid < n_it) bc_dq_load_rows<D>(a, tl, sl, wid, cnt, g, cur);
  for (int k0 = kbeg; k0 < kend; k0 += KSEG) {
    const int nk = min(KSEG, kend - k0), nfull = nk >> 5;
    if (k0 > kbeg) {
      __syncthreads();
      if (wid < n_it) bc_dq_load_rows<D>(a, tl, sl, wid, cnt, g, cur);
    }
    p_stage2<D, false, 64 * NW>(a.v.Ks + (size_t)g * D, a.v.Vs + (size_t)g * D, kstride, k0, (nk + 31) >> 5, Kt, Vt);
    __syncthreads();
    for (int it = wid; it < n_it; it += NW) {
      BcDqRows<D> nxt;
      if (it + NW < n_it) bc_dq_load_rows<D>(a, tl, sl, it + NW, cnt, g, nxt);
      f32x4 acc[D / 16];
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (k0 > kbeg && cur.valid) {  // continue from the partial of the earlier segments
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
          const bf16x4 x = *reinterpret_cast<const bf16x4 *>(a.pdq + (size_t)cur.prow * D + acc_dim(dt, quad));
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[dt][i] = (float)x[i];
        }
      }
#pragma unroll
      for (int t = 0; t < MAXT; ++t)
        if (t < nfull) bc_dq_tile<D, false>(acc, cur, kt + t * P::BYTES, vt + t * P::BYTES, ln, 32 * t, nk, sl2);
      if (nk & 31) bc_dq_tile<D, true>(acc, cur, kt + nfull * P::BYTES, vt + nfull * P::BYTES, ln, 32 * nfull, nk, sl2);
      store_partial_row<D>(a.pdq + (size_t)cur.prow * D, acc, cur.valid);
      cur = nxt;
    }
  }
}

// dQ[tok] = (compression + window part, fp32, by sorted position) + scale * sum over the token's selected blocks, in
// rank order, of the partial dQ (which the block-centric kernel leaves without the softmax scale).  One thread per
// (sorted position, query head, 8 dims).
struct DqMergeArgs {
  const bf16_t *pdq;
  const float *dQp;
  const int32_t *idx, *perm;
  bf16_t *dQ;
  int N, Hq, Hkv, hs, T, D;
  float scale;
};

__global__ __launch_bounds__(256) void m_dq_merge(DqMergeArgs a) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per_row = a.D / 8;
  if (i >= (size_t)a.N * a.Hq * per_row) return;
  const int c8 = (int)(i % per_row), h = (int)(i / per_row % a.Hq), pos = (int)(i / ((size_t)per_row * a.Hq));
  const int g = h / a.hs, hl = h % a.hs, tok = a.perm[pos];
  const int32_t *row = a.idx + ((size_t)tok * a.Hkv + g) * a.T;
  int nv = 0;  // rows are ascending with the -1 padding at the end
  for (int j = 0; j < a.T; ++j) nv += row[j] >= 0 ? 1 : 0;
  const float *base = a.dQp + ((size_t)pos * a.Hq + h) * a.D + 8 * c8;
  const float4 b0 = *reinterpret_cast<const float4 *>(base), b1 = *reinterpret_cast<const float4 *>(base + 4);
  const float part[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const size_t slot0 = ((size_t)pos * a.Hkv + g) * a.T;
#pragma unroll 4
  for (int j = 0; j < nv; ++j) {
    const bf16x8 x = ld8(a.pdq + ((slot0 + j) * a.hs + hl) * a.D + 8 * c8);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += (float)x[e];
  }
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)__builtin_fmaf(a.scale, acc[e], part[e]);
  *reinterpret_cast<bf16x8 *>(a.dQ + ((size_t)tok * a.Hq + h) * a.D + 8 * c8) = o;
}

// Shape of the block-centric kernels per head dimension: wavefronts per workgroup, keys held in LDS at a time.
template <int D> struct BcShape { static constexpr int NW = 8, KSEG = 256; };

// upper bound of the number of chunks: every (KV head, block) list adds at most one partly filled chunk
unsigned chunk_bound(const MfmaView &v) {
  const size_t entries = (size_t)v.N * v.Hkv * v.T;
  return (unsigned)(entries / BC_CHUNK + (size_t)v.Hkv * v.Ns);
}

template <int D>
int launch_slc_forward(const MfmaView &v, const bf16_t *q, const int32_t *idx, const SelIndex &sel, const SlcPartials &part,
                       hipStream_t s) {
  using BS = BcShape<D>;
  static std::once_flag once;  // raise the dynamic LDS limit once per process for this instantiation
  std::call_once(once, [] {
    (void)hipFuncSetAttribute((const void *)m_slc_fwd_bc<D, BS::NW, BS::KSEG>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              160 * 1024);
  });
  BcFwdArgs b{v, q, idx, sel.start, sel.list, sel.bc_chunk_start, sel.bc_order, part.o, part.ml};
  m_slc_fwd_bc<D, BS::NW, BS::KSEG><<<dim3((chunk_bound(v) + 7) / 8 * 8), 64 * BS::NW, bc_lds_bytes<D, BS::KSEG>(), s>>>(b);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

template <int D>
int launch_slc_dq(const MfmaView &v, const BwdBuffers &w, const int32_t *idx, hipStream_t s) {
  using BS = BcShape<D>;
  static std::once_flag once;
  std::call_once(once, [] {
    (void)hipFuncSetAttribute((const void *)m_bwd_dq_bc<D, BS::NW, BS::KSEG>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              160 * 1024);
  });
  const size_t NH = (size_t)v.N * v.Hq;
  BcDqArgs b{v, w.Qs, w.dOg + NH * D, w.lse2s + NH, w.deltag + NH, idx, w.sel.start, w.sel.list, w.sel.bc_chunk_start,
             w.sel.bc_order, w.part.o};
  m_bwd_dq_bc<D, BS::NW, BS::KSEG><<<dim3((chunk_bound(v) + 7) / 8 * 8), 64 * BS::NW, bc_dq_lds_bytes<D, BS::KSEG>(), s>>>(b);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

}  // namespace

int slc_forward_kernel(const MfmaView &v, int D, const void *q, const int32_t *idx, const SelIndex &sel,
                       const SlcPartials &part, hipStream_t s) {
  switch (D) {
    case 32: return launch_slc_forward<32>(v, (const bf16_t *)q, idx, sel, part, s);
    case 64: return launch_slc_forward<64>(v, (const bf16_t *)q, idx, sel, part, s);
    case 128: return launch_slc_forward<128>(v, (const bf16_t *)q, idx, sel, part, s);
    default: return SSA_ERR_UNSUPPORTED;
  }
}

int slc_merge_kernel(const MfmaView &v, int D, const SlcPartials &part, const int32_t *idx, const void *gates,
                     void *out_branch, float *lse, void *out, hipStream_t s) {
  MergeArgs m{part.o, part.ml, idx, (const bf16_t *)gates, (bf16_t *)out_branch, lse, (bf16_t *)out,
              v.N, v.Hq, v.Hkv, v.hs, v.T, D, v.sl2};
  const size_t threads = (size_t)v.N * v.Hq * (D / 8);
  m_slc_merge<<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(m);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

int slc_dq_kernel(const MfmaView &v, int D, const BwdBuffers &w, const int32_t *idx, hipStream_t s) {
  switch (D) {
    case 32: return launch_slc_dq<32>(v, w, idx, s);
    case 64: return launch_slc_dq<64>(v, w, idx, s);
    case 128: return launch_slc_dq<128>(v, w, idx, s);
    default: return SSA_ERR_UNSUPPORTED;
  }
}

int slc_dq_merge_kernel(const MfmaView &v, int D, const BwdBuffers &w, const int32_t *idx, void *dq, hipStream_t s) {
  DqMergeArgs m{w.part.o, w.dQp, idx, v.perm, (bf16_t *)dq, v.N, v.Hq, v.Hkv, v.hs, v.T, D, v.scale};
  const size_t threads = (size_t)v.N * v.Hq * (D / 8);
  m_dq_merge<<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(m);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}
