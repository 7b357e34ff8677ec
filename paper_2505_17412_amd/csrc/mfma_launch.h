// Launch functions of the bf16 MFMA kernels (defined in mfma_fwd.hip / mfma_bwd.hip / mfma_slc.hip), called by
// mfma_path.hip and by one another.
#pragma once
#include "mfma_common.h"

size_t mfma_fwd_lds_bytes(int D, int hs, int s_max);
struct SelIndex;
struct SlcPartials;
int mfma_forward_kernels(const MfmaView &v, int D, const void *q, const void *gates, void *out, float *lse,
                         int32_t *idx, void *out_branch, const SelIndex &sel, const SlcPartials &part, hipStream_t s);

// Inverse of the selection (sel_index.hip): per (KV head, selection block) key = g*Ns + b, the ascending list of sorted
// positions of the tokens that selected it, and the cuts of the lists into work chunks.
struct SelIndex {
  uint32_t *bits;                 // [Hkv*Ns][ceil(N/32)] bit (key, pos): token at pos selected the block
  uint32_t *counts;               // [Hkv*Ns]
  int32_t *start, *list;          // [Hkv*Ns+1], [N*Hkv*T]
  int32_t *chunk_start, *part_row_start;  // [Hkv*Ns+1] each: dK/dV work chunks and partial-sum rows per key
  int32_t *bc_chunk_start;        // [Hkv*Ns+1]: work chunks of the block-centric forward / dQ kernels
  int32_t *order, *bc_order;      // execution order of the chunks of either chunking (chunk ids; see m_chunk_order)
  int chunk_len, bc_chunk_len;    // query tokens per chunk of either kind (at least 256)
};
size_t sel_index_bytes(int N, int Hkv, int T, int Ns);
SelIndex sel_index_carve(void *ws, int N, int Hkv, int T, int Ns, int chunk_len, int bc_chunk_len);
int sel_index_build(const int32_t *idx, const int32_t *perm, const int32_t *slc_start, int N, int Hkv, int T, int Ns,
                    const SelIndex &x, bool want_dkv_order, hipStream_t s);

// Block-centric selection kernels: query tokens per work chunk, and the per-(token, KV head, rank) partial results.
constexpr int BC_CHUNK = 256;
struct SlcPartials {
  bf16_t *o;    // [N][Hkv][T][hs][D]: unnormalised partial output (forward) / partial dQ (backward) per selected block
  float *ml;    // [N][Hkv][T][hs][2]: running maximum (raw score units) and sum of the partial softmax (forward only)
};

// Block-centric selection kernels (mfma_slc.hip), forward: partials per selected block, then the per-token merge that
// also writes the gated sum of eq. (4) (out_branch [3,N,Hq,D]: branches 0 and 2 read, 1 written; lse [3,N,Hq]).
int slc_forward_kernel(const MfmaView &v, int D, const void *q, const int32_t *idx, const SelIndex &sel,
                       const SlcPartials &part, hipStream_t s);
int slc_merge_kernel(const MfmaView &v, int D, const SlcPartials &part, const int32_t *idx, const void *gates,
                     void *out_branch, float *lse, void *out, hipStream_t s);

// Device buffers of the backward pass (carved from the caller's workspace).
struct BwdBuffers {
  float *lse2s, *deltas, *gws;  // [3][N(pos)][Hq]: lse*log2(e), gate*<dO,O_b>, gate
  float *deltag;                // [3][N(pos)][Hq]: <gate*dO as rounded into dOg, O_b>: the delta of the kernels that read dOg
  bf16_t *Qs, *dOg;             // sorted token order: Q [N(pos)][Hq][D]; gate_b * dO [3][N(pos)][Hq][D], one copy per branch b
  float *dKs, *dVs;             // [N(pos)][Hkv][D] token-level gradients in sorted order
  float *dQp;                   // [N(pos)][Hq][D] compression-branch part of dQ (fp32)
  float *dKc, *dVc;             // [q_splits][Nc][Hkv][D] partial gradients of the pooled keys/values
  SelIndex sel;
  float *pK, *pV;               // [max_part_rows][D] per-chunk partial dK/dV of the selection branch
  int max_chunks;               // upper bound of the number of dK/dV chunks
  int q_splits;
  float *dKc_out, *dVc_out;     // [Nc][Hkv][D] or NULL: where the pooled-key/value gradients go instead of being un-pooled
  SlcPartials part;             // partial dQ of the selection branch
};
// Block-centric selection kernels, backward: partial dQ per selected block (w.part.o), then the per-token sum onto the
// fp32 dQ of the other two branches (w.dQp), written to dq.
int slc_dq_kernel(const MfmaView &v, int D, const BwdBuffers &w, const int32_t *idx, hipStream_t s);
int slc_dq_merge_kernel(const MfmaView &v, int D, const BwdBuffers &w, const int32_t *idx, void *dq, hipStream_t s);
int mfma_backward_kernels(const MfmaView &v, int D, const BwdBuffers &w, const void *q, const void *gates,
                          const void *out_branch, const float *lse, const int32_t *idx, const void *dout, void *dq,
                          void *dk, void *dv, void *dgates, const ssa_blocks *blk, int B, hipStream_t s);
