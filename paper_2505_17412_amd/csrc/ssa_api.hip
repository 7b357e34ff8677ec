// C ABI of the SSA library: argument validation and dispatch (see include/ssa.h for the contract).
#include "ssa_internal.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

namespace {

// SSA_FORCE_GENERIC=1 in the environment routes bf16 problems through the fp32-arithmetic kernels as well
// (a debugging aid; both paths run on the GPU).
bool force_generic() {
  static const bool v = [] {
    const char *e = getenv("SSA_FORCE_GENERIC");
    return e && e[0] == '1';
  }();
  return v;
}

int make_ctx(const ssa_params_t *p, const ssa_blocks_t *b, void *stream, ssa_ctx *c) {
  if (!p || !b) return SSA_ERR_NULL;
  if (p->n_tokens < 0 || p->n_batch < 1 || p->topk < 1 || p->topk > 64) return SSA_ERR_BAD_SHAPE;
  if (p->dtype != SSA_BF16 && p->dtype != SSA_F32) return SSA_ERR_BAD_SHAPE;
  if (p->n_heads_q < 1 || p->n_heads_kv < 1 || p->n_heads_q % p->n_heads_kv != 0) return SSA_ERR_BAD_HEADS;
  if (p->head_dim < 8 || p->head_dim > 128 || p->head_dim % 8 != 0) return SSA_ERR_UNSUPPORTED;
  if (p->n_heads_q / p->n_heads_kv > 64) return SSA_ERR_UNSUPPORTED;
  if (p->n_tokens != b->N || p->n_batch != b->B || p->grid != b->G || p->m_cmp != b->m_cmp || p->m_slc != b->m_slc ||
      p->m_win != b->m_win)
    return SSA_ERR_MISMATCH;
  if ((long long)p->n_tokens * p->n_heads_q > 2000000000ll / 3) return SSA_ERR_BAD_SHAPE;
  c->N = p->n_tokens; c->B = p->n_batch; c->Hq = p->n_heads_q; c->Hkv = p->n_heads_kv; c->hs = c->Hq / c->Hkv;
  c->d = p->head_dim; c->T = p->topk; c->dtype = p->dtype;
  c->scale = p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)p->head_dim);
  c->blk = b;
  c->stream = (hipStream_t)stream;
  return SSA_OK;
}

bool use_mfma(const ssa_ctx &c) { return !force_generic() && mfma_supported(c); }

}  // namespace

extern "C" size_t ssa_workspace_bytes(const ssa_params_t *p, const ssa_blocks_t *b, int for_backward) {
  ssa_ctx c;
  if (make_ctx(p, b, nullptr, &c) != SSA_OK) return 0;
  size_t n;
  if (use_mfma(c)) n = for_backward ? mfma_backward_workspace(c) : mfma_forward_workspace(c);
  else n = for_backward ? generic_backward_workspace(c) : generic_forward_workspace(c);
  return n + 256;
}

extern "C" int ssa_forward(const ssa_params_t *p, const ssa_blocks_t *b, const void *q, const void *k, const void *v,
                           const void *gates, void *out, float *lse, int32_t *topk_idx, void *out_branch, void *ws,
                           size_t ws_bytes, void *stream) {
  ssa_ctx c;
  const int rc = make_ctx(p, b, stream, &c);
  if (rc != SSA_OK) return rc;
  if (c.N == 0) return SSA_OK;
  if (!q || !k || !v || !gates || !out) return SSA_ERR_NULL;
  if (!aligned16(q, k, v, gates, out, lse, topk_idx, out_branch)) return SSA_ERR_ALIGNMENT;
  if (!ws || ws_bytes < ssa_workspace_bytes(p, b, 0)) return SSA_ERR_WORKSPACE;
  void *w = (void *)align_up((size_t)ws, 256);
  const size_t wb = ws_bytes - ((size_t)w - (size_t)ws);
  if (use_mfma(c)) return mfma_forward(c, q, k, v, gates, out, lse, topk_idx, out_branch, w, wb);
  return generic_forward(c, q, k, v, gates, out, lse, topk_idx, out_branch, w, wb);
}

extern "C" int ssa_backward(const ssa_params_t *p, const ssa_blocks_t *b, const void *q, const void *k, const void *v,
                            const void *gates, const void *out_branch, const float *lse, const int32_t *topk_idx,
                            const void *dout, void *dq, void *dk, void *dv, void *dgates, void *ws, size_t ws_bytes,
                            void *stream) {
  ssa_ctx c;
  const int rc = make_ctx(p, b, stream, &c);
  if (rc != SSA_OK) return rc;
  if (c.N == 0) return SSA_OK;
  if (!q || !k || !v || !gates || !out_branch || !lse || !topk_idx || !dout || !dq || !dk || !dv || !dgates)
    return SSA_ERR_NULL;
  if (!aligned16(q, k, v, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates)) return SSA_ERR_ALIGNMENT;
  if (!ws || ws_bytes < ssa_workspace_bytes(p, b, 1)) return SSA_ERR_WORKSPACE;
  void *w = (void *)align_up((size_t)ws, 256);
  const size_t wb = ws_bytes - ((size_t)w - (size_t)ws);
  if (use_mfma(c))
    return mfma_backward(c, q, k, v, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates, w, wb);
  return generic_backward(c, q, k, v, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates, w, wb);
}

extern "C" int ssa_forward_pooled(const ssa_params_t *p, const ssa_blocks_t *b, const void *q, const void *k,
                                  const void *v, const void *gates, const void *k_cmp, const void *v_cmp, void *out,
                                  float *lse, int32_t *topk_idx, void *out_branch, void *ws, size_t ws_bytes,
                                  void *stream) {
  ssa_ctx c;
  const int rc = make_ctx(p, b, stream, &c);
  if (rc != SSA_OK) return rc;
  if (!use_mfma(c)) return SSA_ERR_UNSUPPORTED;
  if (c.N == 0) return SSA_OK;
  if (!q || !k || !v || !gates || !k_cmp || !v_cmp || !out) return SSA_ERR_NULL;
  if (!aligned16(q, k, v, gates, k_cmp, v_cmp, out, lse, topk_idx, out_branch)) return SSA_ERR_ALIGNMENT;
  if (!ws || ws_bytes < ssa_workspace_bytes(p, b, 0)) return SSA_ERR_WORKSPACE;
  void *w = (void *)align_up((size_t)ws, 256);
  const size_t wb = ws_bytes - ((size_t)w - (size_t)ws);
  c.kc_in = k_cmp; c.vc_in = v_cmp;
  return mfma_forward(c, q, k, v, gates, out, lse, topk_idx, out_branch, w, wb);
}

extern "C" int ssa_backward_pooled(const ssa_params_t *p, const ssa_blocks_t *b, const void *q, const void *k,
                                   const void *v, const void *gates, const void *k_cmp, const void *v_cmp,
                                   const void *out_branch, const float *lse, const int32_t *topk_idx, const void *dout,
                                   void *dq, void *dk, void *dv, void *dgates, float *dk_cmp, float *dv_cmp, void *ws,
                                   size_t ws_bytes, void *stream) {
  ssa_ctx c;
  const int rc = make_ctx(p, b, stream, &c);
  if (rc != SSA_OK) return rc;
  if (!use_mfma(c) || !mfma_backward_covers(c)) return SSA_ERR_UNSUPPORTED;
  if (c.N == 0) return SSA_OK;
  if (!q || !k || !v || !gates || !k_cmp || !v_cmp || !out_branch || !lse || !topk_idx || !dout || !dq || !dk || !dv ||
      !dgates || !dk_cmp || !dv_cmp)
    return SSA_ERR_NULL;
  if (!aligned16(q, k, v, gates, k_cmp, v_cmp, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates, dk_cmp, dv_cmp))
    return SSA_ERR_ALIGNMENT;
  if (!ws || ws_bytes < ssa_workspace_bytes(p, b, 1)) return SSA_ERR_WORKSPACE;
  void *w = (void *)align_up((size_t)ws, 256);
  const size_t wb = ws_bytes - ((size_t)w - (size_t)ws);
  c.kc_in = k_cmp; c.vc_in = v_cmp; c.dkc_out = dk_cmp; c.dvc_out = dv_cmp;
  return mfma_backward(c, q, k, v, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates, w, wb);
}

extern "C" int ssa_topk_from_scores(const ssa_params_t *p, const ssa_blocks_t *b, const float *scores, int32_t *topk_idx,
                                    void *stream) {
  if (!p || !b) return SSA_ERR_NULL;
  if (p->n_tokens != b->N) return SSA_ERR_MISMATCH;
  if (p->n_heads_kv < 1) return SSA_ERR_BAD_HEADS;
  if (p->topk < 1 || p->topk > 64) return SSA_ERR_BAD_SHAPE;
  if (b->N == 0) return SSA_OK;
  if (!scores || !topk_idx) return SSA_ERR_NULL;
  ssa_ctx c{};
  c.N = b->N; c.Hkv = p->n_heads_kv; c.T = p->topk; c.blk = b; c.stream = (hipStream_t)stream;
  return launch_topk_from_scores(c, scores, topk_idx);
}

extern "C" const char *ssa_error_string(int s) {
  switch (s) {
    case SSA_OK: return "ok";
    case SSA_ERR_NULL: return "a required pointer is NULL";
    case SSA_ERR_BAD_SHAPE: return "bad shape (token/batch count, grid, top-k or dtype out of range)";
    case SSA_ERR_BAD_BLOCK_SIZES: return "block sides must satisfy m_slc > m_cmp and m_cmp | m_slc";
    case SSA_ERR_BAD_HEADS: return "head counts must be positive with Hq divisible by Hkv";
    case SSA_ERR_BAD_OFFSETS: return "batch offsets must rise monotonically from 0 to n_tokens";
    case SSA_ERR_COORD_RANGE: return "a voxel coordinate lies outside [0, grid)";
    case SSA_ERR_WORKSPACE: return "workspace missing or too small";
    case SSA_ERR_UNSUPPORTED: return "unsupported configuration (block side not a power of two, or head_dim)";
    case SSA_ERR_HIP: return "a HIP runtime call failed";
    case SSA_ERR_MISMATCH: return "parameters do not match the blocks handle";
    case SSA_ERR_ALIGNMENT: return "a tensor pointer is not 16-byte aligned";
    default: return "unknown status";
  }
}
