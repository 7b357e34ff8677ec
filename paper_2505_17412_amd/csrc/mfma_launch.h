// Launch functions of the bf16 MFMA kernels (defined in mfma_fwd.hip / mfma_bwd.hip), called by mfma_path.hip.
#pragma once
#include "mfma_common.h"

size_t mfma_fwd_lds_bytes(int D, int hs, int s_max, int T, int Ns);
int mfma_forward_kernels(const MfmaView &v, int D, const void *q, const void *gates, void *out, float *lse,
                         int32_t *idx, void *out_branch, void *order_ws, hipStream_t s);

// Token order of the selection-branch kernels (slc_order.hip): per KV head, the tokens' caller indices ordered so that
// tokens with similar selected sets are neighbours; *order = [Hkv][N] inside `ws`, or NULL when the problem is too
// small to bother (the kernels then walk the sorted order).
constexpr int SLC_ORDER_MIN_TOKENS = 4096;
size_t slc_order_workspace(int N, int Hkv, int Ns);
int slc_order_build(const int32_t *idx, const int32_t *perm, int N, int Hkv, int T, int Ns, void *ws, hipStream_t s,
                    const int32_t **order);

// Device buffers of the backward pass (carved from the caller's workspace).
struct BwdBuffers {
  float *lse2s, *deltas, *gws;  // [3][N(pos)][Hq]: lse*log2(e), gate*<dO,O_b>, gate
  bf16_t *Qs, *dOs;             // [N(pos)][Hq][D]: Q and dO in sorted token order
  float *dKs, *dVs;             // [N(pos)][Hkv][D] token-level gradients in sorted order
  float *dQp;                   // [N(pos)][Hq][D] compression-branch part of dQ (fp32)
  float *dKc, *dVc;             // [q_splits][Nc][Hkv][D] partial gradients of the pooled keys/values
  uint32_t *sel_bits;           // [Hkv*Ns][ceil(N/32)] bit (key, pos): token at pos selected the block
  uint32_t *sel_counts;         // [Hkv*Ns]
  int32_t *sel_start, *sel_list;  // [Hkv*Ns+1], [N*Hkv*T]
  int32_t *chunk_start, *part_row_start;  // [Hkv*Ns+1] each: work chunks and partial-sum rows per (g, block)
  float *pK, *pV;               // [max_part_rows][D] per-chunk partial dK/dV of the selection branch
  int chunk_len, max_chunks;    // query tokens per chunk; upper bound of the number of chunks
  int q_splits;
  float *dKc_out, *dVc_out;     // [Nc][Hkv][D] or NULL: where the pooled-key/value gradients go instead of being un-pooled
  void *order_ws;               // slc_order_workspace() bytes
};
int mfma_backward_kernels(const MfmaView &v, int D, const BwdBuffers &w, const void *q, const void *gates,
                          const void *out_branch, const float *lse, const int32_t *idx, const void *dout, void *dq,
                          void *dk, void *dv, void *dgates, const ssa_blocks *blk, int B, hipStream_t s);
