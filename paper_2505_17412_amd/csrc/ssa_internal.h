// Internal declarations shared by the translation units of the SSA library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/ssa.h"

#define SSA_HIP_TRY(expr)                      \
  do {                                         \
    hipError_t e__ = (expr);                   \
    if (e__ != hipSuccess) return SSA_ERR_HIP; \
  } while (0)

// Rows of zero padding kept after the last token / compressed block of the sorted K,V copies, so that a
// key tile that starts inside the data may read past its end.
constexpr int SSA_KEY_PAD = 256;

struct ssa_blocks {
  int32_t N, B, G, m_cmp, m_slc, m_win, bits;
  int32_t Nc, Ns, Nw;
  int32_t s_max;        // max selection blocks in one item
  int32_t c_max;        // max compression blocks in one item
  int32_t slc_tok_max;  // max tokens in one selection block
  int32_t win_tok_max;  // max tokens in one window
  int32_t cmp_tok_max;  // max tokens in one compression block
  int device;
  int dims;  // 3: voxel-grid partition (Morton order); 1: sequences in caller order (block sizes are token counts)
  void *base;  // single device allocation holding every array below
  int32_t *perm, *inv_perm, *tok_item, *tok_cmp, *tok_slc, *tok_win;
  int32_t *cmp_start, *slc_start, *win_start, *slc_child_start, *cmp_slc, *cmp_batch, *slc_batch;
  int32_t *item_start;  // [B+1] sorted-position range of each batch item (a copy of the batch offsets)
  uint64_t *sorted_keys;  // [N] (batch item << 3*bits) | Morton code, ascending: the token order itself
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// True when every pointer of the list (NULL included) sits on a 16-byte boundary: the kernels read and write tensors
// through 16-byte vector accesses.
template <typename... P> static inline bool aligned16(P... p) { return ((((size_t)p) | ...) & 15) == 0; }

static inline int ilog2_exact(int m) {  // m is a power of two
  int l = 0;
  while ((1 << l) < m) ++l;
  return l;
}

// ---- raw bf16 helpers (round to nearest even), usable on host and device
__host__ __device__ static inline float bf16_to_f32(uint16_t b) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)b << 16;
  return c.f;
}
__host__ __device__ static inline uint16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> struct io;
template <> struct io<float> {
  __device__ static inline float ld(const float *p) { return *p; }
  __device__ static inline void st(float *p, float v) { *p = v; }
  __device__ static inline float round(float v) { return v; }
};
template <> struct io<uint16_t> {
  __device__ static inline float ld(const uint16_t *p) { return bf16_to_f32(*p); }
  __device__ static inline void st(uint16_t *p, float v) { *p = f32_to_bf16(v); }
  __device__ static inline float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};

// ---- resolved problem description handed to the launch functions
struct ssa_ctx {
  int N, B, Hq, Hkv, hs, d, T, dtype;
  float scale;
  const ssa_blocks *blk;
  hipStream_t stream;
  // caller-supplied block-level keys/values [Nc][Hkv][d] replacing the mean pool, and where the gradients w.r.t.
  // them go (fp32 [Nc][Hkv][d]); all NULL in the plain entry points
  const void *kc_in = nullptr, *vc_in = nullptr;
  float *dkc_out = nullptr, *dvc_out = nullptr;
};

// ---- generic (any head_dim / head grouping, fp32 arithmetic) path: generic_kernels.hip
size_t generic_forward_workspace(const ssa_ctx &c);
size_t generic_backward_workspace(const ssa_ctx &c);
int generic_forward(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates, void *out,
                    float *lse, int32_t *topk_idx, void *out_branch, void *ws, size_t ws_bytes);
int generic_backward(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates,
                     const void *out_branch, const float *lse, const int32_t *topk_idx, const void *dout, void *dq,
                     void *dk, void *dv, void *dgates, void *ws, size_t ws_bytes);
int launch_topk_from_scores(const ssa_ctx &c, const float *scores, int32_t *topk_idx);

// ---- bf16 MFMA path: mfma_*.hip
bool mfma_supported(const ssa_ctx &c);
bool mfma_backward_covers(const ssa_ctx &c);  // the key-centric backward kernels cover this head grouping
size_t mfma_forward_workspace(const ssa_ctx &c);
size_t mfma_backward_workspace(const ssa_ctx &c);
int mfma_forward(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates, void *out,
                 float *lse, int32_t *topk_idx, void *out_branch, void *ws, size_t ws_bytes);
int mfma_backward(const ssa_ctx &c, const void *q, const void *k, const void *v, const void *gates,
                  const void *out_branch, const float *lse, const int32_t *topk_idx, const void *dout, void *dq,
                  void *dk, void *dv, void *dgates, void *ws, size_t ws_bytes);

// ---- stable radix sort of (uint64 key, uint32 value) pairs: build_blocks.hip
size_t sort_pairs_aux_bytes(int n);
int sort_pairs(uint64_t *k0, uint32_t *v0, uint64_t *k1, uint32_t *v1, void *aux, int n, int bits, hipStream_t stream);
