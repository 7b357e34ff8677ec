// One full SSA attention layer for gfx950, composed on the host from the library's own entry points: query / key /
// value projections and the gate predictor on the input features, Spatial Sparse Attention (eq. (4)), output
// projection; forward and backward.  Paper: gates are "a linear layer followed by a sigmoid" on the input features
// (text after eq. (4)); the projections are those of any attention layer (Implementation Details: hidden dimension
// 1024, grouped-query attention).  Every arithmetic step runs in the kernels of the parts; this file only lays out the
// saved activations and the workspace and orders the launches on the caller's stream.
#include "linear_internal.h"
#include "profile.h"

namespace {

struct SavedPlan {
  size_t q, k, v, gates, o, ob, lse, idx, total;
};

SavedPlan saved_plan(const ssa_params_t *p) {
  const size_t N = (size_t)p->n_tokens, cq = (size_t)p->n_heads_q * p->head_dim, ckv = (size_t)p->n_heads_kv * p->head_dim;
  SavedPlan s{};
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t r = off; off += align_up(bytes, 256); return r; };
  s.q = take(N * cq * 2);
  s.k = take(N * ckv * 2);
  s.v = take(N * ckv * 2);
  s.gates = take(N * p->n_heads_q * 3 * 2);
  s.o = take(N * cq * 2);
  s.ob = take(3 * N * cq * 2);
  s.lse = take(3 * N * p->n_heads_q * 4);
  s.idx = take(N * p->n_heads_kv * p->topk * 4);
  s.total = off;
  return s;
}

struct BwdPlan {
  size_t d_o, dq, dk, dv, dg, kc, vc, dkc, dvc, scratch, scratch_bytes, total;
};

// Forward workspace: the learned module's block tokens in front of a scratch region shared by the parts.
struct FwdPlan {
  size_t kc, vc, scratch, scratch_bytes, total;
};

// 0: mean pool; 1: learned compression module on keys and values; -1: some but not all of its pointers given
int module_mode(const ssa_layer_weights_t *w) {
  const int n = (w->pe_k != nullptr) + (w->wc_k != nullptr) + (w->bc_k != nullptr) + (w->pe_v != nullptr) +
                (w->wc_v != nullptr) + (w->bc_v != nullptr);
  return n == 0 ? 0 : n == 6 ? 1 : -1;
}

size_t max3(size_t a, size_t b, size_t c) { return a > b ? (a > c ? a : c) : (b > c ? b : c); }

FwdPlan fwd_plan(const ssa_params_t *p, const ssa_blocks_t *b, int Dm) {
  const size_t ckv = (size_t)p->n_heads_kv * p->head_dim;
  FwdPlan w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t r = off; off += align_up(bytes, 256); return r; };
  w.kc = take((size_t)b->Nc * ckv * 2);
  w.vc = take((size_t)b->Nc * ckv * 2);
  w.scratch_bytes = max3(ssa_workspace_bytes(p, b, 0), ssa_gate_workspace_bytes(p, Dm, 0), ssa_compress_workspace_bytes(p, b, 0)) + 256;
  w.scratch = take(w.scratch_bytes);
  w.total = off;
  return w;
}

BwdPlan bwd_plan(const ssa_params_t *p, const ssa_blocks_t *b, int Dm) {
  const size_t N = (size_t)p->n_tokens, cq = (size_t)p->n_heads_q * p->head_dim, ckv = (size_t)p->n_heads_kv * p->head_dim;
  BwdPlan w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t r = off; off += align_up(bytes, 256); return r; };
  w.d_o = take(N * cq * 2);
  w.dq = take(N * cq * 2);
  w.dk = take(N * ckv * 2);
  w.dv = take(N * ckv * 2);
  w.dg = take(N * p->n_heads_q * 3 * 2);
  w.kc = take((size_t)b->Nc * ckv * 2);  // the learned module's block tokens (recomputed) and their gradients
  w.vc = take((size_t)b->Nc * ckv * 2);
  w.dkc = take((size_t)b->Nc * ckv * 4);
  w.dvc = take((size_t)b->Nc * ckv * 4);
  const size_t wt = align_up(cq * Dm * 2, 256) + 2 * align_up(ckv * Dm * 2, 256);  // transposed Wq, Wk, Wv
  const size_t lin = max3(ssa_linear_workspace_bytes(p->n_tokens, (int)cq, Dm, 1), lin_dw_workspace(p->n_tokens, Dm, (int)cq),
                          lin_dw_workspace(p->n_tokens, Dm, (int)ckv));
  const size_t mod = max3(ssa_compress_workspace_bytes(p, b, 0), ssa_compress_workspace_bytes(p, b, 1), 0);
  w.scratch_bytes = max3(max3(wt, lin, mod), ssa_workspace_bytes(p, b, 1), ssa_gate_workspace_bytes(p, Dm, 1)) + 256;
  w.scratch = take(w.scratch_bytes);
  w.total = off;
  return w;
}

int layer_check(const ssa_params_t *p, const ssa_blocks_t *b, int Dm) {
  if (!p || !b) return SSA_ERR_NULL;
  if (p->dtype != SSA_BF16) return SSA_ERR_UNSUPPORTED;
  if (p->n_heads_q < 1 || p->n_heads_kv < 1 || p->head_dim < 1) return SSA_ERR_BAD_HEADS;
  const long long cq = (long long)p->n_heads_q * p->head_dim, ckv = (long long)p->n_heads_kv * p->head_dim;
  if (cq > 16384 || ckv > 16384) return SSA_ERR_UNSUPPORTED;
  int rc = lin_check(p->n_tokens, Dm, (int)cq);
  if (rc == SSA_OK) rc = lin_check(p->n_tokens, Dm, (int)ckv);
  if (rc != SSA_OK) return rc;
  if (p->n_tokens > 0 && ssa_workspace_bytes(p, b, 0) == 0) return SSA_ERR_MISMATCH;  // the attention call would refuse
  if (ssa_gate_workspace_bytes(p, Dm, 0) == 0) return SSA_ERR_UNSUPPORTED;
  return SSA_OK;
}

}  // namespace

extern "C" size_t ssa_layer_saved_bytes(const ssa_params_t *p, size_t *offsets) {
  if (!p || p->n_tokens < 0 || p->n_heads_q < 1 || p->n_heads_kv < 1 || p->head_dim < 1 || p->topk < 1) return 0;
  const SavedPlan s = saved_plan(p);
  if (offsets) {
    const size_t o[8] = {s.q, s.k, s.v, s.gates, s.o, s.ob, s.lse, s.idx};
    for (int i = 0; i < 8; ++i) offsets[i] = o[i];
  }
  return s.total + 256;
}

extern "C" size_t ssa_layer_workspace_bytes(const ssa_params_t *p, const ssa_blocks_t *b, int32_t d_model, int for_backward) {
  if (layer_check(p, b, d_model) != SSA_OK) return 0;
  if (for_backward) return bwd_plan(p, b, d_model).total + 256;
  return fwd_plan(p, b, d_model).total + 256;
}

extern "C" int ssa_layer_forward(const ssa_params_t *p, const ssa_blocks_t *b, int32_t d_model, const void *x,
                                 const ssa_layer_weights_t *w, void *y, void *saved_, size_t saved_bytes, void *ws,
                                 size_t ws_bytes, void *stream) {
  const int rc0 = layer_check(p, b, d_model);
  if (rc0 != SSA_OK) return rc0;
  if (p->n_tokens == 0) return SSA_OK;
  if (!x || !w || !y || !saved_) return SSA_ERR_NULL;
  if (!w->wq || !w->wk || !w->wv || !w->wg || !w->bg || !w->wo) return SSA_ERR_NULL;
  if (!aligned16(x, y)) return SSA_ERR_ALIGNMENT;  // the weights are checked by the parts
  if (saved_bytes < ssa_layer_saved_bytes(p, nullptr)) return SSA_ERR_WORKSPACE;
  if (!ws || ws_bytes < ssa_layer_workspace_bytes(p, b, d_model, 0)) return SSA_ERR_WORKSPACE;
  const int mode = module_mode(w);
  if (mode < 0) return SSA_ERR_NULL;
  if (mode == 1 && ssa_compress_workspace_bytes(p, b, 0) == 0) return SSA_ERR_UNSUPPORTED;
  const SavedPlan s = saved_plan(p);
  const FwdPlan pl = fwd_plan(p, b, d_model);
  char *sv = (char *)align_up((size_t)saved_, 256);
  char *wsb = (char *)align_up((size_t)ws, 256);
  char *scratch = wsb + pl.scratch;
  const int N = p->n_tokens, cq = p->n_heads_q * p->head_dim, ckv = p->n_heads_kv * p->head_dim;
  int rc = ssa_linear_forward(N, d_model, cq, x, w->wq, w->bq, sv + s.q, stream);
  if (rc == SSA_OK) rc = ssa_linear_forward(N, d_model, ckv, x, w->wk, w->bk, sv + s.k, stream);
  if (rc == SSA_OK) rc = ssa_linear_forward(N, d_model, ckv, x, w->wv, w->bv, sv + s.v, stream);
  if (rc == SSA_OK) rc = ssa_gate_forward(p, d_model, x, w->wg, w->bg, sv + s.gates, scratch, pl.scratch_bytes, stream);
  if (rc == SSA_OK && mode == 1) {
    const ssa_cmp_weights_t ck{w->pe_k, w->wc_k, w->bc_k}, cv{w->pe_v, w->wc_v, w->bc_v};
    rc = ssa_compress_forward(p, b, sv + s.k, &ck, wsb + pl.kc, scratch, pl.scratch_bytes, stream);
    if (rc == SSA_OK) rc = ssa_compress_forward(p, b, sv + s.v, &cv, wsb + pl.vc, scratch, pl.scratch_bytes, stream);
    if (rc == SSA_OK)
      rc = ssa_forward_pooled(p, b, sv + s.q, sv + s.k, sv + s.v, sv + s.gates, wsb + pl.kc, wsb + pl.vc, sv + s.o,
                              (float *)(sv + s.lse), (int32_t *)(sv + s.idx), sv + s.ob, scratch, pl.scratch_bytes, stream);
  } else if (rc == SSA_OK) {
    rc = ssa_forward(p, b, sv + s.q, sv + s.k, sv + s.v, sv + s.gates, sv + s.o, (float *)(sv + s.lse), (int32_t *)(sv + s.idx),
                     sv + s.ob, scratch, pl.scratch_bytes, stream);
  }
  if (rc == SSA_OK) rc = ssa_linear_forward(N, cq, d_model, sv + s.o, w->wo, w->bo, y, stream);
  return rc;
}

extern "C" int ssa_layer_backward(const ssa_params_t *p, const ssa_blocks_t *b, int32_t d_model, const void *x,
                                  const ssa_layer_weights_t *w, const void *saved_, const void *dy, void *dx,
                                  const ssa_layer_grads_t *g, void *ws_, size_t ws_bytes, void *stream) {
  const int rc0 = layer_check(p, b, d_model);
  if (rc0 != SSA_OK) return rc0;
  if (!w || !g) return SSA_ERR_NULL;
  if (!g->dwq || !g->dwk || !g->dwv || !g->dwg || !g->dbg || !g->dwo) return SSA_ERR_NULL;
  const int mode = module_mode(w);
  if (mode < 0) return SSA_ERR_NULL;
  if (mode == 1 && (!g->dpe_k || !g->dwc_k || !g->dbc_k || !g->dpe_v || !g->dwc_v || !g->dbc_v)) return SSA_ERR_NULL;
  if (mode == 1 && ssa_compress_workspace_bytes(p, b, 1) == 0) return SSA_ERR_UNSUPPORTED;
  const ssa_cmp_weights_t ck{w->pe_k, w->wc_k, w->bc_k}, cv{w->pe_v, w->wc_v, w->bc_v};
  hipStream_t st = (hipStream_t)stream;
  const int N = p->n_tokens, cq = p->n_heads_q * p->head_dim, ckv = p->n_heads_kv * p->head_dim;
  if (N == 0) {  // no tokens: every parameter gradient is zero (the parts write the zeros)
    int rc = ssa_linear_backward(0, cq, d_model, nullptr, nullptr, nullptr, nullptr, g->dwo, g->dbo, nullptr, 0, stream);
    if (rc == SSA_OK) rc = ssa_linear_backward(0, d_model, cq, nullptr, nullptr, nullptr, nullptr, g->dwq, g->dbq, nullptr, 0, stream);
    if (rc == SSA_OK) rc = ssa_linear_backward(0, d_model, ckv, nullptr, nullptr, nullptr, nullptr, g->dwk, g->dbk, nullptr, 0, stream);
    if (rc == SSA_OK) rc = ssa_linear_backward(0, d_model, ckv, nullptr, nullptr, nullptr, nullptr, g->dwv, g->dbv, nullptr, 0, stream);
    if (rc == SSA_OK) rc = ssa_gate_backward(p, d_model, nullptr, nullptr, nullptr, nullptr, nullptr, g->dwg, g->dbg, nullptr, 0, stream);
    if (rc == SSA_OK && mode == 1)
      rc = ssa_compress_backward(p, b, nullptr, &ck, nullptr, nullptr, g->dpe_k, g->dwc_k, g->dbc_k, nullptr, 0, stream);
    if (rc == SSA_OK && mode == 1)
      rc = ssa_compress_backward(p, b, nullptr, &cv, nullptr, nullptr, g->dpe_v, g->dwc_v, g->dbc_v, nullptr, 0, stream);
    return rc;
  }
  if (!x || !saved_ || !dy || !dx) return SSA_ERR_NULL;
  if (!aligned16(x, dy, dx, w->wq, w->wk, w->wv, g->dwq, g->dwk, g->dwv, g->dbq, g->dbk, g->dbv)) return SSA_ERR_ALIGNMENT;
  if (!w->wq || !w->wk || !w->wv || !w->wg || !w->wo) return SSA_ERR_NULL;
  if (!ws_ || ws_bytes < ssa_layer_workspace_bytes(p, b, d_model, 1)) return SSA_ERR_WORKSPACE;
  const SavedPlan s = saved_plan(p);
  const BwdPlan pl = bwd_plan(p, b, d_model);
  const char *sv = (const char *)align_up((size_t)saved_, 256);
  char *ws = (char *)align_up((size_t)ws_, 256);
  void *d_o = ws + pl.d_o, *dq = ws + pl.dq, *dk = ws + pl.dk, *dv = ws + pl.dv, *dg = ws + pl.dg;
  char *scratch = ws + pl.scratch;
  // output projection: dO and its parameter gradients
  int rc = ssa_linear_backward(N, cq, d_model, sv + s.o, w->wo, dy, d_o, g->dwo, g->dbo, scratch, pl.scratch_bytes, stream);
  if (rc != SSA_OK) return rc;
  if (mode == 1) {
    // the block tokens are recomputed rather than saved (two small launches); their gradients flow back through
    // the module onto dk and dv
    void *kc = ws + pl.kc, *vc = ws + pl.vc;
    float *dkc = (float *)(ws + pl.dkc), *dvc = (float *)(ws + pl.dvc);
    rc = ssa_compress_forward(p, b, sv + s.k, &ck, kc, scratch, pl.scratch_bytes, stream);
    if (rc == SSA_OK) rc = ssa_compress_forward(p, b, sv + s.v, &cv, vc, scratch, pl.scratch_bytes, stream);
    if (rc == SSA_OK)
      rc = ssa_backward_pooled(p, b, sv + s.q, sv + s.k, sv + s.v, sv + s.gates, kc, vc, sv + s.ob, (const float *)(sv + s.lse),
                               (const int32_t *)(sv + s.idx), d_o, dq, dk, dv, dg, dkc, dvc, scratch, pl.scratch_bytes, stream);
    if (rc == SSA_OK)
      rc = ssa_compress_backward(p, b, sv + s.k, &ck, dkc, dk, g->dpe_k, g->dwc_k, g->dbc_k, scratch, pl.scratch_bytes, stream);
    if (rc == SSA_OK)
      rc = ssa_compress_backward(p, b, sv + s.v, &cv, dvc, dv, g->dpe_v, g->dwc_v, g->dbc_v, scratch, pl.scratch_bytes, stream);
  } else {
    rc = ssa_backward(p, b, sv + s.q, sv + s.k, sv + s.v, sv + s.gates, sv + s.ob, (const float *)(sv + s.lse),
                      (const int32_t *)(sv + s.idx), d_o, dq, dk, dv, dg, scratch, pl.scratch_bytes, stream);
  }
  if (rc != SSA_OK) return rc;
  {
    ProfScope ps(PROF_LINEAR_BWD, st);
    lin_dw(N, d_model, cq, x, dq, g->dwq, g->dbq, scratch, st);
    lin_dw(N, d_model, ckv, x, dk, g->dwk, g->dbk, scratch, st);
    lin_dw(N, d_model, ckv, x, dv, g->dwv, g->dbv, scratch, st);
    // dx = dq Wq + dk Wk + dv Wv in one launch over the three contractions
    char *wtq = scratch, *wtk = wtq + align_up((size_t)cq * d_model * 2, 256), *wtv = wtk + align_up((size_t)ckv * d_model * 2, 256);
    lin_transpose_w(w->wq, cq, d_model, wtq, st);
    lin_transpose_w(w->wk, ckv, d_model, wtk, st);
    lin_transpose_w(w->wv, ckv, d_model, wtv, st);
    const void *Xs[3] = {dq, dk, dv}, *Ws[3] = {wtq, wtk, wtv};
    const int Ks[3] = {cq, ckv, ckv};
    rc = lin_nt_multi(3, Xs, Ws, Ks, nullptr, N, d_model, dx, st);
    if (rc != SSA_OK) return rc;
  }
  // gate predictor: its data gradient is added onto dx
  rc = ssa_gate_backward(p, d_model, x, w->wg, sv + s.gates, dg, dx, g->dwg, g->dbg, scratch, pl.scratch_bytes, stream);
  if (rc != SSA_OK) return rc;
  SSA_HIP_TRY(hipGetLastError());
  return SSA_OK;
}
