// Generic SSA path: fp32 arithmetic on the vector ALUs, one wavefront per (token, query head) or per key row.
// Serves SSA_F32 problems and every shape the bf16 MFMA kernels do not cover.  Same mathematics as the MFMA
// path (paper eq. (2)-(6), Algorithm 1, window paragraph), written for clarity, not speed.
#include "ssa_internal.h"
#include "profile.h"
#include "topk_device.h"
#include "mfma_launch.h"

namespace {

constexpr int WAVE = 64;

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

struct BlkView {
  const int32_t *perm, *tok_item, *tok_cmp, *tok_win, *cmp_start, *slc_start, *win_start, *slc_child_start, *cmp_batch,
      *slc_batch;
};

static BlkView view_of(const ssa_blocks *b) {
  return BlkView{b->perm, b->tok_item, b->tok_cmp, b->tok_win, b->cmp_start, b->slc_start, b->win_start,
                 b->slc_child_start, b->cmp_batch, b->slc_batch};
}

// Sorted fp32 copies of K,V and their per-compression-block means (eq. (5), mean pool over active tokens).
template <typename T>
__global__ void g_sort_pool(const T *__restrict__ K, const T *__restrict__ V, BlkView bv, int row /*Hkv*d*/,
                            float *__restrict__ Ks, float *__restrict__ Vs, float *__restrict__ Kc,
                            float *__restrict__ Vc) {
  const int c = blockIdx.x;
  const int b = bv.cmp_start[c], e = bv.cmp_start[c + 1];
  const float inv = 1.0f / (float)(e - b);
  for (int i = threadIdx.x; i < row; i += blockDim.x) {
    float sk = 0.f, sv = 0.f;
    for (int pos = b; pos < e; ++pos) {
      const size_t src = (size_t)bv.perm[pos] * row + i;
      const float kk = io<T>::ld(K + src), vv = io<T>::ld(V + src);
      Ks[(size_t)pos * row + i] = kk;
      Vs[(size_t)pos * row + i] = vv;
      sk += kk;
      sv += vv;
    }
    // rounded to the element type: a bf16 problem sees the same pooled rows here as in the matrix-core kernels, whose
    // forward may have produced the lse this path's backward is given
    Kc[(size_t)c * row + i] = io<T>::round(sk * inv);
    Vc[(size_t)c * row + i] = io<T>::round(sv * inv);
  }
}

// Online-softmax state of one query row spread over a wavefront (lanes hold output dims lane and lane+64).
struct RowState {
  float m, l, a0, a1;
};

__device__ inline void attend_range(RowState &st, const float *qs /*LDS, pre-scaled*/, float *ps /*LDS[64]*/,
                                    const float *__restrict__ Kb, const float *__restrict__ Vb, int kb, int ke, int Hkv,
                                    int g, int d) {
  const int lane = threadIdx.x;
  for (int k0 = kb; k0 < ke; k0 += WAVE) {
    const int key = k0 + lane;
    float s = -INFINITY;
    if (key < ke) {
      const float *kr = Kb + ((size_t)key * Hkv + g) * d;
      float acc = 0.f;
      for (int i = 0; i < d; ++i) acc += qs[i] * kr[i];
      s = acc;
    }
    const float mn = fmaxf(st.m, wave_max(s));
    const float p = key < ke ? __expf(s - mn) : 0.f;
    const float alpha = __expf(st.m - mn);  // exp(-inf) = 0 on the first tile
    st.l = st.l * alpha + wave_sum(p);
    st.a0 *= alpha;
    st.a1 *= alpha;
    st.m = mn;
    ps[lane] = p;
    __syncthreads();
    const int n = min(WAVE, ke - k0);
    for (int kk = 0; kk < n; ++kk) {
      const float *vr = Vb + ((size_t)(k0 + kk) * Hkv + g) * d;
      const float pv = ps[kk];
      if (lane < d) st.a0 += pv * vr[lane];
      if (lane + WAVE < d) st.a1 += pv * vr[lane + WAVE];
    }
    __syncthreads();
  }
}

// branch: 0 compression, 1 selection, 2 window.  One wavefront per (sorted position, query head).
template <typename T>
__global__ void g_attn_fwd(int branch, const T *__restrict__ Q, BlkView bv, const int32_t *__restrict__ idx, int N,
                           int Hq, int Hkv, int d, int Tk, float scale, const float *__restrict__ Kb,
                           const float *__restrict__ Vb, T *__restrict__ Ob, float *__restrict__ lse) {
  __shared__ float qs[128];
  __shared__ float ps[WAVE];
  const int pos = blockIdx.x / Hq, h = blockIdx.x % Hq, hs = Hq / Hkv, g = h / hs, lane = threadIdx.x;
  const int tok = bv.perm[pos];
  for (int i = lane; i < d; i += WAVE) qs[i] = io<T>::ld(Q + ((size_t)tok * Hq + h) * d + i) * scale;
  __syncthreads();
  RowState st{-INFINITY, 0.f, 0.f, 0.f};
  if (branch == 0) {
    const int item = bv.tok_item[pos];
    attend_range(st, qs, ps, Kb, Vb, bv.cmp_batch[item], bv.cmp_batch[item + 1], Hkv, g, d);
  } else if (branch == 2) {
    const int w = bv.tok_win[pos];
    attend_range(st, qs, ps, Kb, Vb, bv.win_start[w], bv.win_start[w + 1], Hkv, g, d);
  } else {
    const int32_t *row = idx + ((size_t)tok * Hkv + g) * Tk;
    for (int j = 0; j < Tk; ++j) {
      const int b = row[j];
      if (b < 0) break;
      attend_range(st, qs, ps, Kb, Vb, bv.slc_start[b], bv.slc_start[b + 1], Hkv, g, d);
    }
  }
  const float inv = st.l > 0.f ? 1.0f / st.l : 0.f;
  T *o = Ob + (((size_t)branch * N + tok) * Hq + h) * d;
  if (lane < d) io<T>::st(o + lane, st.a0 * inv);
  if (lane + WAVE < d) io<T>::st(o + lane + WAVE, st.a1 * inv);
  if (lane == 0) lse[((size_t)branch * N + tok) * Hq + h] = st.l > 0.f ? st.m + __logf(st.l) : -INFINITY;
}

// Selection scores (eq. (6)) and top-k.  One wavefront per (sorted position, KV head).
template <typename T>
__global__ void g_scores_topk(const T *__restrict__ Q, BlkView bv, int N, int Hq, int Hkv, int d, int Tk, float scale,
                              const float *__restrict__ Kc, const float *__restrict__ lse_cmp /*[N,Hq] caller order*/,
                              int32_t *__restrict__ idx, int s_max) {
  extern __shared__ float smem[];
  const int hs = Hq / Hkv;
  float *S = smem;                       // [s_max]
  float *qs = S + s_max;                 // [hs][d]
  float *ls = qs + hs * d;               // [hs]
  uint32_t *sel = (uint32_t *)(ls + hs); // [(s_max+31)/32]
  const int pos = blockIdx.x / Hkv, g = blockIdx.x % Hkv, lane = threadIdx.x;
  const int tok = bv.perm[pos], item = bv.tok_item[pos];
  for (int i = lane; i < hs * d; i += WAVE) qs[i] = io<T>::ld(Q + ((size_t)tok * Hq + g * hs) * d + i) * scale;
  for (int i = lane; i < hs; i += WAVE) ls[i] = lse_cmp[(size_t)tok * Hq + g * hs + i];
  __syncthreads();
  const int s0 = bv.slc_batch[item], s1 = bv.slc_batch[item + 1];
  for (int b = s0 + lane; b < s1; b += WAVE) {
    float acc = 0.f;
    for (int c = bv.slc_child_start[b]; c < bv.slc_child_start[b + 1]; ++c) {
      const float *kr = Kc + ((size_t)c * Hkv + g) * d;
      for (int hl = 0; hl < hs; ++hl) {
        float s = 0.f;
        for (int i = 0; i < d; ++i) s += qs[hl * d + i] * kr[i];
        acc += __expf(s - ls[hl]);
      }
    }
    S[b - s0] = acc;
  }
  __syncthreads();
  topk_wave(S, s1 - s0, Tk, s0, idx + ((size_t)tok * Hkv + g) * Tk, sel);
}

__global__ void g_topk_from_scores(const float *__restrict__ scores, BlkView bv, int N, int Hkv, int Tk, int s_max,
                                   const int32_t *__restrict__ inv_perm, int32_t *__restrict__ idx) {
  extern __shared__ float smem[];
  float *S = smem;
  uint32_t *sel = (uint32_t *)(S + s_max);
  const int tok = blockIdx.x / Hkv, g = blockIdx.x % Hkv;
  const int item = bv.tok_item[inv_perm[tok]];
  const int s0 = bv.slc_batch[item], n = bv.slc_batch[item + 1] - s0;
  for (int i = threadIdx.x; i < n; i += WAVE) S[i] = scores[((size_t)tok * Hkv + g) * s_max + i];
  __syncthreads();
  topk_wave(S, n, Tk, s0, idx + ((size_t)tok * Hkv + g) * Tk, sel);
}

// eq. (4): out = sum_b gate_b * out_b
template <typename T>
__global__ void g_combine(const T *__restrict__ Ob, const T *__restrict__ gates, size_t N, int Hq, int d,
                          T *__restrict__ out) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = N * Hq * d;
  if (i >= total) return;
  const size_t th = i / d;
  float acc = 0.f;
  for (int b = 0; b < 3; ++b) acc += io<T>::ld(gates + th * 3 + b) * io<T>::ld(Ob + (size_t)b * total + i);
  io<T>::st(out + i, acc);
}

// dgates[t,h,b] = <dO, O_b>; delta[b,t,h] = gate_b * dgates  (= <gate_b*dO, O_b>, the softmax-backward row term)
template <typename T>
__global__ void g_bwd_pre(const T *__restrict__ dO, const T *__restrict__ Ob, const T *__restrict__ gates, size_t N,
                          int Hq, int d, T *__restrict__ dgates, float *__restrict__ delta) {
  const size_t th = blockIdx.x;  // token*Hq + head, caller order
  const int lane = threadIdx.x;
  for (int b = 0; b < 3; ++b) {
    float acc = 0.f;
    for (int i = lane; i < d; i += WAVE)
      acc += io<T>::ld(dO + th * d + i) * io<T>::ld(Ob + ((size_t)b * N * Hq + th) * d + i);
    acc = wave_sum(acc);
    if (lane == 0) {
      io<T>::st(dgates + th * 3 + b, acc);
      delta[(size_t)b * N * Hq + th] = acc * io<T>::ld(gates + th * 3 + b);
    }
  }
}

struct BwdRow {
  float dq0, dq1;
};

__device__ inline void attend_range_bwd(BwdRow &r, const float *qs /*unscaled*/, const float *gb, float *dss, float lse,
                                        float delta, float scale, const float *__restrict__ Kb,
                                        const float *__restrict__ Vb, int kb, int ke, int Hkv, int g, int d) {
  const int lane = threadIdx.x;
  for (int k0 = kb; k0 < ke; k0 += WAVE) {
    const int key = k0 + lane;
    float ds = 0.f;
    if (key < ke) {
      const float *kr = Kb + ((size_t)key * Hkv + g) * d;
      const float *vr = Vb + ((size_t)key * Hkv + g) * d;
      float s = 0.f, dp = 0.f;
      for (int i = 0; i < d; ++i) {
        s += qs[i] * kr[i];
        dp += gb[i] * vr[i];
      }
      ds = __expf(s * scale - lse) * (dp - delta) * scale;
    }
    dss[lane] = ds;
    __syncthreads();
    const int n = min(WAVE, ke - k0);
    for (int kk = 0; kk < n; ++kk) {
      const size_t row = ((size_t)(k0 + kk) * Hkv + g) * d;
      const float dv = dss[kk];
      if (lane < d) r.dq0 += dv * Kb[row + lane];
      if (lane + WAVE < d) r.dq1 += dv * Kb[row + lane + WAVE];
    }
    __syncthreads();
  }
}

// dQ of all three branches for one (sorted position, head): query-centric, the keys of each branch in turn.
template <typename T>
__global__ void g_attn_bwd_dq(const T *__restrict__ Q, const T *__restrict__ dO, const T *__restrict__ gates, BlkView bv,
                              const int32_t *__restrict__ idx, int N, int Hq, int Hkv, int d, int Tk, float scale,
                              const float *__restrict__ Ks, const float *__restrict__ Vs, const float *__restrict__ Kc,
                              const float *__restrict__ Vc, const float *__restrict__ lse, const float *__restrict__ delta,
                              T *__restrict__ dQ) {
  __shared__ float qs[128], go[128], gb[128], dss[WAVE];
  const int pos = blockIdx.x / Hq, h = blockIdx.x % Hq, hs = Hq / Hkv, g = h / hs, lane = threadIdx.x;
  const int tok = bv.perm[pos];
  const size_t th = (size_t)tok * Hq + h;
  for (int i = lane; i < d; i += WAVE) {
    qs[i] = io<T>::ld(Q + th * d + i);
    go[i] = io<T>::ld(dO + th * d + i);
  }
  BwdRow r{0.f, 0.f};
  for (int branch = 0; branch < 3; ++branch) {
    __syncthreads();
    const float w = io<T>::ld(gates + th * 3 + branch);
    for (int i = lane; i < d; i += WAVE) gb[i] = w * go[i];
    __syncthreads();
    const float l = lse[(size_t)branch * N * Hq + th], dl = delta[(size_t)branch * N * Hq + th];
    if (branch == 0) {
      const int item = bv.tok_item[pos];
      attend_range_bwd(r, qs, gb, dss, l, dl, scale, Kc, Vc, bv.cmp_batch[item], bv.cmp_batch[item + 1], Hkv, g, d);
    } else if (branch == 2) {
      const int wdw = bv.tok_win[pos];
      attend_range_bwd(r, qs, gb, dss, l, dl, scale, Ks, Vs, bv.win_start[wdw], bv.win_start[wdw + 1], Hkv, g, d);
    } else {
      const int32_t *row = idx + ((size_t)tok * Hkv + g) * Tk;
      for (int j = 0; j < Tk; ++j) {
        const int b = row[j];
        if (b < 0) break;
        attend_range_bwd(r, qs, gb, dss, l, dl, scale, Ks, Vs, bv.slc_start[b], bv.slc_start[b + 1], Hkv, g, d);
      }
    }
  }
  if (lane < d) io<T>::st(dQ + th * d + lane, r.dq0);
  if (lane + WAVE < d) io<T>::st(dQ + th * d + lane + WAVE, r.dq1);
}

// dK, dV of one key row (sorted token, or compression block when `pooled`) and KV head: key-centric, so that every sum
// runs in one fixed order and no floating-point atomic is needed (results are the same from run to run).  The queries
// that attend the key: for a token, the tokens of its window (window branch), then the tokens whose selected sets hold
// its selection block, in ascending sorted position (selection branch; lists from the inverse selection index); for a
// compression block, every token of its batch item.  64 query rows (token x head of the group) at a time: each lane
// forms its row's probability and dS, then the lanes, now standing for output dims, add the 64 contributions in order.
template <typename T>
__global__ void g_attn_bwd_dkv(int pooled, const T *__restrict__ Q, const T *__restrict__ dO, const T *__restrict__ gates,
                               BlkView bv, const int32_t *__restrict__ tok_slc, const int32_t *__restrict__ item_start,
                               const int32_t *__restrict__ sel_start, const int32_t *__restrict__ sel_list, int N, int B,
                               int Ns, int Hq, int Hkv, int d, float scale, const float *__restrict__ Kr,
                               const float *__restrict__ Vr, const float *__restrict__ lse,
                               const float *__restrict__ delta, float *__restrict__ dK, float *__restrict__ dV) {
  __shared__ float ks[128], vs[128], ps[WAVE], dss[WAVE];
  __shared__ size_t qth[WAVE];
  const int key = blockIdx.x, g = blockIdx.y, hs = Hq / Hkv, lane = threadIdx.x;
  const size_t krow = ((size_t)key * Hkv + g) * d;
  for (int i = lane; i < d; i += WAVE) {
    ks[i] = Kr[krow + i];
    vs[i] = Vr[krow + i];
  }
  __syncthreads();
  float dk0 = 0.f, dk1 = 0.f, dv0 = 0.f, dv1 = 0.f;
  const size_t NH = (size_t)N * Hq;
  // queries e = 0 .. count*hs-1: token number e / hs of the list, head g*hs + e % hs
  auto run = [&](int branch, const int32_t *list, int first, int count) {
    for (int e0 = 0; e0 < count * hs; e0 += WAVE) {
      const int e = e0 + lane;
      float p = 0.f, ds = 0.f;
      size_t th = 0;
      if (e < count * hs) {
        const int pos = list ? list[first + e / hs] : first + e / hs;
        th = (size_t)bv.perm[pos] * Hq + g * hs + e % hs;
        const float w = io<T>::ld(gates + th * 3 + branch);
        float s = 0.f, dp = 0.f;
        for (int i = 0; i < d; ++i) {
          s += io<T>::ld(Q + th * d + i) * ks[i];
          dp += io<T>::ld(dO + th * d + i) * vs[i];
        }
        const float pr = __expf(s * scale - lse[branch * NH + th]);
        ds = pr * (w * dp - delta[branch * NH + th]) * scale;
        p = pr * w;
      }
      ps[lane] = p;
      dss[lane] = ds;
      qth[lane] = th;
      __syncthreads();
      const int n = min(WAVE, count * hs - e0);
      for (int kk = 0; kk < n; ++kk) {
        const size_t row = qth[kk] * d;
        if (lane < d) {
          dv0 += ps[kk] * io<T>::ld(dO + row + lane);
          dk0 += dss[kk] * io<T>::ld(Q + row + lane);
        }
        if (lane + WAVE < d) {
          dv1 += ps[kk] * io<T>::ld(dO + row + lane + WAVE);
          dk1 += dss[kk] * io<T>::ld(Q + row + lane + WAVE);
        }
      }
      __syncthreads();
    }
  };
  if (pooled) {
    int item = 0;
    while (item + 1 < B && key >= bv.cmp_batch[item + 1]) ++item;
    run(0, nullptr, item_start[item], item_start[item + 1] - item_start[item]);
  } else {
    const int w = bv.tok_win[key];
    run(2, nullptr, bv.win_start[w], bv.win_start[w + 1] - bv.win_start[w]);
    const int sk = g * Ns + tok_slc[key];
    run(1, sel_list, sel_start[sk], sel_start[sk + 1] - sel_start[sk]);
  }
  if (lane < d) { dK[krow + lane] = dk0; dV[krow + lane] = dv0; }
  if (lane + WAVE < d) { dK[krow + lane + WAVE] = dk1; dV[krow + lane + WAVE] = dv1; }
}

// dK[tok] = dKs[pos] + dKc[cmp(pos)] / count (gradient of the mean pool), scattered back to caller order.
template <typename T>
__global__ void g_unpool_scatter(BlkView bv, size_t N, int row, const float *__restrict__ dKs,
                                 const float *__restrict__ dVs, const float *__restrict__ dKc,
                                 const float *__restrict__ dVc, T *__restrict__ dK, T *__restrict__ dV) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N * row) return;
  const size_t pos = i / row;
  const int f = (int)(i % row);
  const int c = bv.tok_cmp[pos];
  const float inv = 1.0f / (float)(bv.cmp_start[c + 1] - bv.cmp_start[c]);
  const size_t dst = (size_t)bv.perm[pos] * row + f;
  io<T>::st(dK + dst, dKs[i] + dKc[(size_t)c * row + f] * inv);
  io<T>::st(dV + dst, dVs[i] + dVc[(size_t)c * row + f] * inv);
}

struct GenericPlan {
  size_t ks, vs, kc, vc, ob, lse, idx, delta, dks, dvs, dkc, dvc, sel, total;
};

GenericPlan plan(const ssa_ctx &c, bool bwd) {
  GenericPlan p{};
  const size_t esz = c.dtype == SSA_F32 ? 4 : 2;
  const size_t kv = align_up((size_t)c.N * c.Hkv * c.d * 4 + 4, 256);
  const size_t kvc = align_up((size_t)c.blk->Nc * c.Hkv * c.d * 4 + 4, 256);
  size_t off = 0;
  auto take = [&](size_t n) { size_t r = off; off += align_up(n, 256); return r; };
  p.ks = take(kv); p.vs = take(kv); p.kc = take(kvc); p.vc = take(kvc);
  if (!bwd) {
    p.ob = take((size_t)3 * c.N * c.Hq * c.d * esz + 4);
    p.lse = take((size_t)3 * c.N * c.Hq * 4 + 4);
    p.idx = take((size_t)c.N * c.Hkv * c.T * 4 + 4);
  } else {
    p.delta = take((size_t)3 * c.N * c.Hq * 4 + 4);
    p.dks = take(kv); p.dvs = take(kv); p.dkc = take(kvc); p.dvc = take(kvc);
    p.sel = take(sel_index_bytes(c.N, c.Hkv, c.T, c.blk->Ns));
  }
  p.total = off;
  return p;
}

size_t scores_lds_bytes(const ssa_ctx &c) {
  return ((size_t)c.blk->s_max + (size_t)c.hs * c.d + c.hs + ((size_t)c.blk->s_max + 31) / 32 + 4) * 4;
}

template <typename T>
int forward_t(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates, void *out, float *lse,
              int32_t *topk_idx, void *out_branch, char *ws) {
  const GenericPlan p = plan(c, false);
  const BlkView bv = view_of(c.blk);
  float *Ks = (float *)(ws + p.ks), *Vs = (float *)(ws + p.vs), *Kc = (float *)(ws + p.kc), *Vc = (float *)(ws + p.vc);
  T *Ob = out_branch ? (T *)out_branch : (T *)(ws + p.ob);
  float *L = lse ? lse : (float *)(ws + p.lse);
  int32_t *I = topk_idx ? topk_idx : (int32_t *)(ws + p.idx);
  const int N = c.N, row = c.Hkv * c.d;
  if (scores_lds_bytes(c) > 60000) return SSA_ERR_UNSUPPORTED;
  g_sort_pool<T><<<c.blk->Nc, 256, 0, c.stream>>>((const T *)k, (const T *)v, bv, row, Ks, Vs, Kc, Vc);
  g_attn_fwd<T><<<N * c.Hq, WAVE, 0, c.stream>>>(0, (const T *)q, bv, nullptr, N, c.Hq, c.Hkv, c.d, c.T, c.scale, Kc, Vc, Ob, L);
  g_scores_topk<T><<<N * c.Hkv, WAVE, scores_lds_bytes(c), c.stream>>>((const T *)q, bv, N, c.Hq, c.Hkv, c.d, c.T, c.scale, Kc, L, I,
                                                                      c.blk->s_max);
  g_attn_fwd<T><<<N * c.Hq, WAVE, 0, c.stream>>>(1, (const T *)q, bv, I, N, c.Hq, c.Hkv, c.d, c.T, c.scale, Ks, Vs, Ob, L);
  g_attn_fwd<T><<<N * c.Hq, WAVE, 0, c.stream>>>(2, (const T *)q, bv, nullptr, N, c.Hq, c.Hkv, c.d, c.T, c.scale, Ks, Vs, Ob, L);
  const size_t total = (size_t)N * c.Hq * c.d;
  g_combine<T><<<(unsigned)((total + 255) / 256), 256, 0, c.stream>>>(Ob, (const T *)gates, (size_t)N, c.Hq, c.d, (T *)out);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

template <typename T>
int backward_t(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates, const void *out_branch,
               const float *lse, const int32_t *topk_idx, const void *dout, void *dq, void *dk, void *dv, void *dgates,
               char *ws) {
  const GenericPlan p = plan(c, true);
  const BlkView bv = view_of(c.blk);
  float *Ks = (float *)(ws + p.ks), *Vs = (float *)(ws + p.vs), *Kc = (float *)(ws + p.kc), *Vc = (float *)(ws + p.vc);
  float *delta = (float *)(ws + p.delta);
  float *dKs = (float *)(ws + p.dks), *dVs = (float *)(ws + p.dvs), *dKc = (float *)(ws + p.dkc), *dVc = (float *)(ws + p.dvc);
  const int N = c.N, row = c.Hkv * c.d;
  g_sort_pool<T><<<c.blk->Nc, 256, 0, c.stream>>>((const T *)k, (const T *)v, bv, row, Ks, Vs, Kc, Vc);
  g_bwd_pre<T><<<N * c.Hq, WAVE, 0, c.stream>>>((const T *)dout, (const T *)out_branch, (const T *)gates, (size_t)N, c.Hq, c.d,
                                                (T *)dgates, delta);
  g_attn_bwd_dq<T><<<N * c.Hq, WAVE, 0, c.stream>>>((const T *)q, (const T *)dout, (const T *)gates, bv, topk_idx, N, c.Hq, c.Hkv,
                                                    c.d, c.T, c.scale, Ks, Vs, Kc, Vc, lse, delta, (T *)dq);
  const SelIndex sel = sel_index_carve(ws + p.sel, N, c.Hkv, c.T, c.blk->Ns, 1024, 1024);
  const int rc = sel_index_build(topk_idx, c.blk->perm, c.blk->slc_start, N, c.Hkv, c.T, c.blk->Ns, sel, false, c.stream);
  if (rc != SSA_OK) return rc;
  g_attn_bwd_dkv<T><<<dim3(N, c.Hkv), WAVE, 0, c.stream>>>(0, (const T *)q, (const T *)dout, (const T *)gates, bv, c.blk->tok_slc,
                                                          c.blk->item_start, sel.start, sel.list, N, c.B, c.blk->Ns, c.Hq, c.Hkv,
                                                          c.d, c.scale, Ks, Vs, lse, delta, dKs, dVs);
  g_attn_bwd_dkv<T><<<dim3(c.blk->Nc, c.Hkv), WAVE, 0, c.stream>>>(1, (const T *)q, (const T *)dout, (const T *)gates, bv,
                                                                  c.blk->tok_slc, c.blk->item_start, sel.start, sel.list, N, c.B,
                                                                  c.blk->Ns, c.Hq, c.Hkv, c.d, c.scale, Kc, Vc, lse, delta, dKc,
                                                                  dVc);
  const size_t total = (size_t)N * row;
  g_unpool_scatter<T><<<(unsigned)((total + 255) / 256), 256, 0, c.stream>>>(bv, (size_t)N, row, dKs, dVs, dKc, dVc, (T *)dk,
                                                                            (T *)dv);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

}  // namespace

size_t generic_forward_workspace(const ssa_ctx &c) { return plan(c, false).total; }
size_t generic_backward_workspace(const ssa_ctx &c) { return plan(c, true).total; }

int generic_forward(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates, void *out,
                    float *lse, int32_t *topk_idx, void *out_branch, void *ws, size_t ws_bytes) {
  if (ws_bytes < plan(c, false).total) return SSA_ERR_WORKSPACE;
  if (c.N == 0) return SSA_OK;
  ProfScope ps(PROF_GENERIC, c.stream);
  return c.dtype == SSA_F32
             ? forward_t<float>(c, q, k, v, gates, out, lse, topk_idx, out_branch, (char *)ws)
             : forward_t<uint16_t>(c, q, k, v, gates, out, lse, topk_idx, out_branch, (char *)ws);
}

int generic_backward(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates,
                     const void *out_branch, const float *lse, const int32_t *topk_idx, const void *dout, void *dq,
                     void *dk, void *dv, void *dgates, void *ws, size_t ws_bytes) {
  if (ws_bytes < plan(c, true).total) return SSA_ERR_WORKSPACE;
  if (c.N == 0) return SSA_OK;
  ProfScope ps(PROF_GENERIC, c.stream);
  return c.dtype == SSA_F32
             ? backward_t<float>(c, q, k, v, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates, (char *)ws)
             : backward_t<uint16_t>(c, q, k, v, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates, (char *)ws);
}

int launch_topk_from_scores(const ssa_ctx &c, const float *scores, int32_t *topk_idx) {
  if (c.N == 0) return SSA_OK;
  const int s_max = c.blk->s_max;
  const size_t lds = ((size_t)s_max + ((size_t)s_max + 31) / 32 + 4) * 4;
  if (lds > 60000) return SSA_ERR_UNSUPPORTED;
  g_topk_from_scores<<<c.N * c.Hkv, WAVE, lds, c.stream>>>(scores, view_of(c.blk), c.N, c.Hkv, c.T, s_max, c.blk->inv_perm,
                                                          topk_idx);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}
