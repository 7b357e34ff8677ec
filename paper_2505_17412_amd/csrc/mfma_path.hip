// bf16 MFMA path: workspace layout, K/V preparation (sort, transpose, mean pool) and launch sequence.
#include "mfma_common.h"
#include "mfma_launch.h"
#include "profile.h"

namespace {

struct Tail { bf16_t *p; size_t begin, end; };  // element range to clear
struct Tails { Tail t[4]; };

__global__ void m_zero_tails(Tails ts) {
  const Tail t = ts.t[blockIdx.y];
  if (!t.p) return;
  for (size_t i = t.begin + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < t.end; i += (size_t)gridDim.x * blockDim.x)
    t.p[i] = 0;
}

struct PrepOut { bf16_t *Ks, *Vs, *Kc, *Vc; };

// One workgroup per compression block: gathers its tokens' K,V rows into sorted order and writes the block mean
// (eq. (5), mean pool over the active tokens).
__global__ void m_prep(const bf16_t *__restrict__ K, const bf16_t *__restrict__ V, const int32_t *__restrict__ perm,
                       const int32_t *__restrict__ cmp_start, int Hkv, int D, PrepOut o) {
  const int c = blockIdx.x, row = Hkv * D;
  const int b = cmp_start[c], e = cmp_start[c + 1];
  const float inv = 1.0f / (float)(e - b);
  for (int f = threadIdx.x; f < row; f += blockDim.x) {
    float sk = 0.f, sv = 0.f;
    for (int pos = b; pos < e; ++pos) {
      const size_t src = (size_t)perm[pos] * row + f;
      const bf16_t kk = K[src], vv = V[src];
      o.Ks[(size_t)pos * row + f] = kk;
      o.Vs[(size_t)pos * row + f] = vv;
      sk += bf16_to_f32(kk);
      sv += bf16_to_f32(vv);
    }
    const bf16_t kc = f32_to_bf16(sk * inv), vc = f32_to_bf16(sv * inv);
    o.Kc[(size_t)c * row + f] = kc;
    o.Vc[(size_t)c * row + f] = vc;
  }
}

// The same with 16-byte accesses, for rows of R8 = Hkv*D/8 pieces with R8 dividing the 128 threads: thread t keeps
// piece t % R8 of tokens b + t/R8, b + t/R8 + 128/R8, ...; the 128/R8 partial sums of a piece meet in LDS and are
// added in a fixed order.
__global__ __launch_bounds__(128) void m_prep8(const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
                                               const int32_t *__restrict__ perm, const int32_t *__restrict__ cmp_start,
                                               int R8, PrepOut o) {
  __shared__ float part[2][128][8];
  const int c = blockIdx.x, b = cmp_start[c], e = cmp_start[c + 1];
  const int seg = threadIdx.x % R8, grp = threadIdx.x / R8, ngrp = 128 / R8;
  float sk[8], sv[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) sk[j] = sv[j] = 0.f;
  for (int pos = b + grp; pos < e; pos += ngrp) {
    const size_t src = ((size_t)perm[pos] * R8 + seg) * 8, dst = ((size_t)pos * R8 + seg) * 8;
    const bf16x8 kk = ld8(K + src), vv = ld8(V + src);
    *reinterpret_cast<bf16x8 *>(o.Ks + dst) = kk;
    *reinterpret_cast<bf16x8 *>(o.Vs + dst) = vv;
#pragma unroll
    for (int j = 0; j < 8; ++j) { sk[j] += (float)kk[j]; sv[j] += (float)vv[j]; }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) { part[0][threadIdx.x][j] = sk[j]; part[1][threadIdx.x][j] = sv[j]; }
  __syncthreads();
  if ((int)threadIdx.x < 2 * R8) {
    const int arr = threadIdx.x / R8, sg = threadIdx.x % R8;
    const float inv = 1.0f / (float)(e - b);
    bf16x8 out;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float t = 0.f;
      for (int gi = 0; gi < ngrp; ++gi) t += part[arr][gi * R8 + sg][j];
      out[j] = (__bf16)(t * inv);
    }
    *reinterpret_cast<bf16x8 *>((arr == 0 ? o.Kc : o.Vc) + ((size_t)c * R8 + sg) * 8) = out;
  }
}

size_t padded_rows(int n) { return align_up((size_t)n, 8) + SSA_KEY_PAD; }

struct FwdPlan { size_t ks, vs, kc, vc, ob, lse, idx, sel, po, pml, total; };

FwdPlan fwd_plan(const ssa_ctx &c) {
  FwdPlan p{};
  const size_t row = (size_t)c.Hkv * c.d * 2;
  size_t off = 0;
  auto take = [&](size_t n) { size_t r = off; off += align_up(n, 256); return r; };
  p.ks = take(padded_rows(c.N) * row); p.vs = take(padded_rows(c.N) * row);
  p.kc = take(padded_rows(c.blk->Nc) * row); p.vc = take(padded_rows(c.blk->Nc) * row);
  p.ob = take((size_t)3 * c.N * c.Hq * c.d * 2);
  p.lse = take((size_t)3 * c.N * c.Hq * 4);
  p.idx = take((size_t)c.N * c.Hkv * c.T * 4);
  p.sel = take(sel_index_bytes(c.N, c.Hkv, c.T, c.blk->Ns));
  const size_t slots = (size_t)c.N * c.Hkv * c.T * c.hs;  // one partial row per (token, query head, selected block)
  p.po = take(slots * c.d * 2);
  p.pml = take(slots * 2 * 4);
  p.total = off;
  return p;
}

MfmaView make_view(const ssa_ctx &c) {
  const ssa_blocks *b = c.blk;
  MfmaView v{};
  v.perm = b->perm; v.tok_item = b->tok_item; v.tok_win = b->tok_win;
  v.cmp_start = b->cmp_start; v.slc_start = b->slc_start; v.win_start = b->win_start;
  v.cmp_slc = b->cmp_slc; v.cmp_batch = b->cmp_batch;
  v.slc_batch = b->slc_batch; v.item_start = b->item_start;
  v.N = c.N; v.Nc = b->Nc; v.Ns = b->Ns; v.Hq = c.Hq; v.Hkv = c.Hkv; v.hs = c.hs; v.T = c.T; v.s_max = b->s_max;
  v.scale = c.scale; v.sl2 = c.scale * LOG2E;
  return v;
}

int run_prep(const ssa_ctx &c, const void *k, const void *v, const PrepOut &o) {
  ProfScope ps(PROF_PREP, c.stream);
  const size_t row = (size_t)c.Hkv * c.d;
  const size_t nt = padded_rows(c.N) * row, nc = padded_rows(c.blk->Nc) * row;
  const size_t t0 = (size_t)(c.N / 8) * 8 * row, c0 = (size_t)(c.blk->Nc / 8) * 8 * row;
  Tails ts{{{o.Ks, t0, nt}, {o.Vs, t0, nt}, {o.Kc, c0, nc}, {o.Vc, c0, nc}}};
  m_zero_tails<<<dim3(8, 4), 256, 0, c.stream>>>(ts);
  const int r8 = c.Hkv * c.d / 8;
  if ((c.Hkv * c.d) % 8 == 0 && r8 <= 64 && 128 % r8 == 0)
    m_prep8<<<c.blk->Nc, 128, 0, c.stream>>>((const bf16_t *)k, (const bf16_t *)v, c.blk->perm, c.blk->cmp_start, r8, o);
  else
    m_prep<<<c.blk->Nc, 128, 0, c.stream>>>((const bf16_t *)k, (const bf16_t *)v, c.blk->perm, c.blk->cmp_start, c.Hkv, c.d, o);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

// Caller-supplied block-level keys/values take the place of the mean-pooled rows (the zero padding behind them stays).
int override_pooled(const ssa_ctx &c, const PrepOut &o) {
  if (!c.kc_in) return SSA_OK;
  const size_t bytes = (size_t)c.blk->Nc * c.Hkv * c.d * sizeof(bf16_t);
  SSA_HIP_TRY(hipMemcpyAsync(o.Kc, c.kc_in, bytes, hipMemcpyDeviceToDevice, c.stream));
  SSA_HIP_TRY(hipMemcpyAsync(o.Vc, c.vc_in, bytes, hipMemcpyDeviceToDevice, c.stream));
  return SSA_OK;
}

struct BwdPlan {
  size_t ks, vs, kc, vc, lse2s, deltas, gws, deltag, qs, dos, dqp, dks, dvs, dkc, dvc, sel, pk, pv, pdq, total;
  int q_splits, chunk_len, max_chunks;
};

constexpr int DKV_WG_KEYS = 128;  // keys per workgroup of the dK/dV kernels (4 waves x 2 blocks of 16)

BwdPlan bwd_plan(const ssa_ctx &c) {
  BwdPlan p{};
  const ssa_blocks *b = c.blk;
  const size_t row = (size_t)c.Hkv * c.d;
  const int tiles = (b->c_max + DKV_WG_KEYS - 1) / DKV_WG_KEYS;
  const long long wgs = (long long)c.B * (tiles > 0 ? tiles : 1) * c.Hkv;
  long long sp = (2048 + wgs - 1) / wgs;  // about 2048 workgroups: four rounds of two per compute unit
  p.q_splits = (int)(sp < 1 ? 1 : (sp > 64 ? 64 : sp));
  size_t off = 0;
  auto take = [&](size_t n) { size_t r = off; off += align_up(n, 256); return r; };
  p.ks = take(padded_rows(c.N) * row * 2); p.vs = take(padded_rows(c.N) * row * 2);
  p.kc = take(padded_rows(b->Nc) * row * 2); p.vc = take(padded_rows(b->Nc) * row * 2);
  const size_t nh = (size_t)3 * c.N * c.Hq * 4;
  p.lse2s = take(nh); p.deltas = take(nh); p.gws = take(nh); p.deltag = take(nh);
  p.qs = take((size_t)c.N * c.Hq * c.d * 2); p.dos = take((size_t)3 * c.N * c.Hq * c.d * 2);
  p.dqp = take((size_t)c.N * c.Hq * c.d * 4);
  p.dks = take((size_t)c.N * row * 4); p.dvs = take((size_t)c.N * row * 4);
  p.dkc = take((size_t)p.q_splits * b->Nc * row * 4); p.dvc = take((size_t)p.q_splits * b->Nc * row * 4);
  const size_t keys = (size_t)c.Hkv * b->Ns;
  p.sel = take(sel_index_bytes(c.N, c.Hkv, c.T, b->Ns));
  // selection-branch work chunks: every (g, block) list is cut into pieces of chunk_len query tokens whose partial
  // dK/dV are summed afterwards in a fixed order.  Bounds: chunks <= entries/chunk_len + keys; partial rows <=
  // slc_tok_max * entries/chunk_len + N*Hkv.  chunk_len grows until the partial sums fit in about 1 GiB.
  const size_t entries = (size_t)c.N * c.Hkv * c.T;
  p.chunk_len = 1024;
  size_t rows;
  for (;;) {
    rows = (size_t)b->slc_tok_max * (entries / p.chunk_len + 1) + (size_t)c.N * c.Hkv;
    if (rows * c.d * 8 <= ((size_t)1 << 30) || p.chunk_len >= (1 << 20)) break;
    p.chunk_len *= 2;
  }
  p.max_chunks = (int)(entries / p.chunk_len + keys + 1);
  p.pk = take(rows * c.d * 4); p.pv = take(rows * c.d * 4);
  p.pdq = take((size_t)c.N * c.Hkv * c.T * c.hs * c.d * 2);  // one partial dQ row per (token, query head, selected block)
  p.total = off;
  return p;
}

// (every backward kernel takes the same head groupings as the forward ones: a 32-row tile holds 32/h_s token slots)
bool mfma_bwd_supported(const ssa_ctx &c) { return c.hs == 1 || c.hs == 2 || c.hs == 4 || c.hs == 8 || c.hs == 16; }

}  // namespace

bool mfma_backward_covers(const ssa_ctx &c) { return mfma_bwd_supported(c); }

bool mfma_supported(const ssa_ctx &c) {
  if (c.dtype != SSA_BF16) return false;
  if (c.d != 32 && c.d != 64 && c.d != 128) return false;
  if (c.hs != 1 && c.hs != 2 && c.hs != 4 && c.hs != 8 && c.hs != 16) return false;
  // the kernels index their staged arrays with 32-bit element offsets
  if ((unsigned long long)(c.N + 2 * SSA_KEY_PAD) * c.Hq * c.d >= (1ull << 31)) return false;
  if (mfma_fwd_lds_bytes(c.d, c.hs, c.blk->s_max) > 150 * 1024) return false;
  // rows of the per-(token, head, selected block) partial arrays are numbered in 32 bits, list entries in int
  if ((unsigned long long)c.N * c.Hq * c.T >= (1ull << 32)) return false;
  if ((unsigned long long)c.N * c.Hkv * c.T >= (1ull << 31)) return false;
  return true;
}

size_t mfma_forward_workspace(const ssa_ctx &c) { return fwd_plan(c).total; }
size_t mfma_backward_workspace(const ssa_ctx &c) {
  return mfma_bwd_supported(c) ? bwd_plan(c).total : generic_backward_workspace(c);
}

int mfma_backward(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates,
                  const void *out_branch, const float *lse, const int32_t *topk_idx, const void *dout, void *dq,
                  void *dk, void *dv, void *dgates, void *ws_, size_t ws_bytes) {
  if (!mfma_bwd_supported(c)) {  // head groupings the key-centric kernels do not cover
    return generic_backward(c, q, k, v, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates, ws_, ws_bytes);
  }
  const BwdPlan p = bwd_plan(c);
  if (ws_bytes < p.total) return SSA_ERR_WORKSPACE;
  char *ws = (char *)ws_;
  PrepOut o{};
  o.Ks = (bf16_t *)(ws + p.ks); o.Vs = (bf16_t *)(ws + p.vs);
  o.Kc = (bf16_t *)(ws + p.kc); o.Vc = (bf16_t *)(ws + p.vc);
  int rc = run_prep(c, k, v, o);
  if (rc != SSA_OK) return rc;
  rc = override_pooled(c, o);
  if (rc != SSA_OK) return rc;
  MfmaView view = make_view(c);
  view.Ks = o.Ks; view.Vs = o.Vs; view.Kc = o.Kc; view.Vc = o.Vc;
  BwdBuffers w{};
  w.dKc_out = c.dkc_out; w.dVc_out = c.dvc_out;
  w.lse2s = (float *)(ws + p.lse2s); w.deltas = (float *)(ws + p.deltas); w.gws = (float *)(ws + p.gws);
  w.deltag = (float *)(ws + p.deltag);
  w.Qs = (bf16_t *)(ws + p.qs); w.dOg = (bf16_t *)(ws + p.dos); w.dQp = (float *)(ws + p.dqp);
  w.dKs = (float *)(ws + p.dks); w.dVs = (float *)(ws + p.dvs); w.dKc = (float *)(ws + p.dkc); w.dVc = (float *)(ws + p.dvc);
  w.sel = sel_index_carve(ws + p.sel, c.N, c.Hkv, c.T, c.blk->Ns, p.chunk_len, BC_CHUNK);
  w.q_splits = p.q_splits;
  w.pK = (float *)(ws + p.pk); w.pV = (float *)(ws + p.pv); w.max_chunks = p.max_chunks;
  w.part = SlcPartials{(bf16_t *)(ws + p.pdq), nullptr};
  return mfma_backward_kernels(view, c.d, w, q, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates, c.blk, c.B,
                               c.stream);
}

int mfma_forward(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates, void *out,
                 float *lse, int32_t *topk_idx, void *out_branch, void *ws_, size_t ws_bytes) {
  const FwdPlan p = fwd_plan(c);
  if (ws_bytes < p.total) return SSA_ERR_WORKSPACE;
  char *ws = (char *)ws_;
  PrepOut o{};
  o.Ks = (bf16_t *)(ws + p.ks); o.Vs = (bf16_t *)(ws + p.vs); o.Kc = (bf16_t *)(ws + p.kc); o.Vc = (bf16_t *)(ws + p.vc);
  int rc = run_prep(c, k, v, o);
  if (rc != SSA_OK) return rc;
  rc = override_pooled(c, o);
  if (rc != SSA_OK) return rc;
  MfmaView view = make_view(c);
  view.Ks = o.Ks; view.Vs = o.Vs; view.Kc = o.Kc; view.Vc = o.Vc;
  const SelIndex sel = sel_index_carve(ws + p.sel, c.N, c.Hkv, c.T, c.blk->Ns, 1024, BC_CHUNK);
  const SlcPartials part{(bf16_t *)(ws + p.po), (float *)(ws + p.pml)};
  return mfma_forward_kernels(view, c.d, q, gates, out, lse ? lse : (float *)(ws + p.lse),
                              topk_idx ? topk_idx : (int32_t *)(ws + p.idx), out_branch ? out_branch : (void *)(ws + p.ob),
                              sel, part, c.stream);
}
