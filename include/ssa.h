/*
 * ssa.h -- C ABI of the MI355X (gfx950) Spatial Sparse Attention library.
 *
 * Spatial Sparse Attention (SSA; paper Sec. "Spatial Sparse Attention", eq. (4)): for every token t and
 * query head h,
 *     o[t,h] = w_cmp * Attn(q, K_cmp, V_cmp) + w_slc * Attn(q, K_slc(t), V_slc(t)) + w_win * Attn(q, K_win(t), V_win(t))
 * where each Attn is softmax attention (eq. (2)-(3)) over a key set defined by 3D blocks of the voxel grid:
 *   cmp: one mean-pooled key/value per non-empty m_cmp^3 block of the token's batch item (eq. (5), mean pool);
 *   slc: all tokens of the T selection blocks (m_slc^3) with the largest score, the score of a block being the
 *        sum of the compression-attention probabilities of its child compression blocks, summed over the
 *        query heads that share a KV head (eq. (6)); ties go to the lowest block id (Algorithm 1 consumes the
 *        resulting index tensor I);
 *   win: all tokens of the token's own m_win^3 window (window paragraph).
 *
 * General conventions
 *   - Every pointer marked "dev" is device memory on the current HIP device; "host" is host memory.
 *   - All tensors are dense, row-major, in the CALLER'S token order.  Query head h uses KV head h / (Hq/Hkv).
 *   - dtype selects the element type of q,k,v,gates,out,out_branch,dout,dq,dk,dv,dgates: SSA_BF16 (2 bytes,
 *     bfloat16) or SSA_F32.  lse is always float, indices are int32.
 *   - The caller owns every tensor and the workspace.  The library owns only ssa_blocks_t.
 *   - Every tensor pointer must sit on a 16-byte boundary (the kernels use 16-byte vector accesses); otherwise
 *     SSA_ERR_ALIGNMENT.  Workspaces may start anywhere: the library aligns inside them.
 *   - ssa_forward / ssa_backward enqueue work on `stream` (a hipStream_t passed as void*) and return without
 *     synchronising; they never allocate.  ssa_build_blocks allocates the handle's arrays and synchronises
 *     the stream once to learn the block counts.
 *   - Return value: 0 on success, a negative ssa_status_t otherwise.  On a validation error nothing is
 *     launched and no output is written.
 */
#ifndef SSA_H_
#define SSA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ssa_blocks ssa_blocks_t; /* opaque: sorted token order + block start arrays (device) */

typedef enum { SSA_BF16 = 0, SSA_F32 = 1 } ssa_dtype_t;

typedef enum {
  SSA_OK = 0,
  SSA_ERR_NULL = -1,            /* a required pointer is NULL */
  SSA_ERR_BAD_SHAPE = -2,       /* n_tokens < 0, n_batch < 1, grid < 1 or > 1024, topk < 1 or > 64, bad dtype */
  SSA_ERR_BAD_BLOCK_SIZES = -3, /* m_slc <= m_cmp or m_slc % m_cmp != 0 or a side < 1 */
  SSA_ERR_BAD_HEADS = -4,       /* Hq % Hkv != 0 or a count < 1 */
  SSA_ERR_BAD_OFFSETS = -5,     /* batch_offsets not monotone from 0 to n_tokens */
  SSA_ERR_COORD_RANGE = -6,     /* a coordinate outside [0, grid) */
  SSA_ERR_WORKSPACE = -7,       /* workspace NULL or smaller than ssa_workspace_bytes() */
  SSA_ERR_UNSUPPORTED = -8,     /* block side not a power of two; head_dim not a multiple of 8 or > 128 */
  SSA_ERR_HIP = -9,             /* a HIP runtime call failed */
  SSA_ERR_MISMATCH = -10,       /* params disagree with the ones the blocks handle was built with */
  SSA_ERR_ALIGNMENT = -11       /* a tensor pointer is not 16-byte aligned */
} ssa_status_t;

typedef struct {
  int32_t n_tokens, n_batch, grid;         /* N, B, G: coordinates lie in [0,G)^3                         */
  int32_t m_cmp, m_slc, m_win, topk;       /* block sides (powers of two, m_cmp | m_slc, m_slc > m_cmp), T */
  int32_t n_heads_q, n_heads_kv, head_dim; /* Hq, Hkv (Hq % Hkv == 0), d (multiple of 8, <= 128)          */
  int32_t dtype;                           /* ssa_dtype_t                                                 */
  float scale;                             /* softmax scale; <= 0 means 1/sqrt(d) (eq. (3))               */
} ssa_params_t;

/* Which array ssa_blocks_export copies out (all int32). */
typedef enum {
  SSA_ARR_PERM = 0,            /* [N]     sorted position -> caller index                                    */
  SSA_ARR_INV_PERM = 1,        /* [N]     caller index -> sorted position                                    */
  SSA_ARR_CMP_START = 2,       /* [Nc+1]  first sorted position of each compression block                    */
  SSA_ARR_SLC_START = 3,       /* [Ns+1]  same for selection blocks: the array C of Algorithm 1              */
  SSA_ARR_WIN_START = 4,       /* [Nw+1]  same for windows                                                   */
  SSA_ARR_SLC_CHILD_START = 5, /* [Ns+1]  compression-block range of each selection block                    */
  SSA_ARR_CMP_BATCH = 6,       /* [B+1]   compression-block range of each batch item                         */
  SSA_ARR_SLC_BATCH = 7,       /* [B+1]   selection-block range of each batch item                           */
  SSA_ARR_TOK_WIN = 8          /* [N]     window id of the token at each sorted position                     */
} ssa_array_t;

/*
 * Block partition, token sort and block start arrays (paper: "we divide the 3D space into subgrids of size
 * m^3 ... tokens residing in the same subgrid are grouped into one block"; "sort the input tokens based on
 * their block indices, then compute the starting index C of each block"; Algorithm 1, Require + line 2).
 *
 * Block ids are dense ranks of (batch item, Morton code of floor(coord/m)) among non-empty blocks, Morton
 * interleaving x -> bit 3i+2, y -> 3i+1, z -> 3i.  Tokens are ordered by (item, full-resolution Morton code),
 * equal voxels by caller index.  Results are bit-exact and deterministic.
 *
 *   params        host; n_tokens, n_batch, grid, m_cmp, m_slc, m_win are read (head fields are ignored)
 *   coords        dev int32 [N,3] voxel coordinates (x,y,z), caller order
 *   batch_offsets dev int32 [B+1], batch_offsets[0]=0, nondecreasing, batch_offsets[B]=N
 *   stream        hipStream_t
 *   out           host; receives a handle to free with ssa_blocks_destroy
 * Errors: NULL, BAD_SHAPE, BAD_BLOCK_SIZES, UNSUPPORTED (before any launch); BAD_OFFSETS, COORD_RANGE (found
 * on the device, reported after the synchronisation; no handle is returned); HIP.
 */
int ssa_build_blocks(const ssa_params_t *params, const int32_t *coords, const int32_t *batch_offsets,
                     void *stream, ssa_blocks_t **out);

/*
 * The same handle for a one-dimensional partition (the paper's remark that its 3D partition takes the place of the
 * 1D blocks of sequence models): batch item i is a sequence of batch_offsets[i+1]-batch_offsets[i] tokens in the
 * caller's order, and a block is a run of m_cmp / m_slc / m_win consecutive tokens counted from the start of the
 * sequence (the last block of a sequence may be shorter).  m_cmp, m_slc, m_win are token counts here, any values
 * with m_slc a proper multiple of m_cmp; params->grid is not read (but must be passed unchanged to the other calls).
 * The token order is the caller's (PERM is the identity).  Every attention entry point accepts the handle;
 * the learned compression module (a convolution on the voxel grid) returns SSA_ERR_UNSUPPORTED for it.
 *
 *   params, batch_offsets, stream, out: as for ssa_build_blocks
 * Errors: NULL, BAD_SHAPE, BAD_BLOCK_SIZES (before any launch); BAD_OFFSETS (found on the device before the
 * partition is built; no handle is returned); HIP.
 */
int ssa_build_blocks_1d(const ssa_params_t *params, const int32_t *batch_offsets, void *stream, ssa_blocks_t **out);

/* Number of non-empty compression / selection / window blocks (host ints; any may be NULL). */
int ssa_blocks_counts(const ssa_blocks_t *blocks, int32_t *n_cmp, int32_t *n_slc, int32_t *n_win);

/* Largest number of selection blocks in one batch item (the row length S_max of ssa_topk_from_scores). */
int ssa_blocks_max_slc_per_item(const ssa_blocks_t *blocks, int32_t *s_max);

/* Copy one index array to dst_dev (dev, `bytes` must be at least its size) on `stream`. */
int ssa_blocks_export(const ssa_blocks_t *blocks, int which, void *dst_dev, size_t bytes, void *stream);

/* Free the handle and its device arrays (NULL is allowed). */
void ssa_blocks_destroy(ssa_blocks_t *blocks);

/*
 * Bytes of device workspace ssa_forward (for_backward == 0) or ssa_backward (!= 0) needs; 0 on bad input.
 * How it scales (bf16 matrix-core path; N tokens, Hq/Hkv heads, head_dim d, top-k T, Ns selection blocks): both passes
 * keep one bf16 partial result per (token, query head, selected block), N*Hq*T*d*2 bytes (2.0 GB at the benchmark
 * shape N = 62k, Hq = 16, T = 16, d = 64; the forward adds N*Hq*T*8 bytes of softmax statistics), and the inverse of the
 * selection: a bit matrix of Hkv*Ns*N/8 bytes plus N*Hkv*T*4 bytes of lists.  Backward adds sorted copies of q and of
 * gate*dout, one per branch (4*N*Hq*d*2 bytes), an fp32 partial dq (N*Hq*d*4 bytes) and up to about 1 GiB of per-chunk
 * partial dk/dv sums.
 */
size_t ssa_workspace_bytes(const ssa_params_t *params, const ssa_blocks_t *blocks, int for_backward);

/*
 * SSA forward (eq. (4); compression eq. (5); selection score eq. (6) and top-k; Algorithm 1; window
 * paragraph).
 *   q        dev [N,Hq,d]      k, v   dev [N,Hkv,d]      gates  dev [N,Hq,3], order (cmp, slc, win)
 *   out      dev [N,Hq,d]      written
 *   lse      dev float [3,N,Hq] or NULL: natural-log log-sum-exp of each branch's scaled logits (Algorithm 1's l)
 *   topk_idx dev int32 [N,Hkv,T] or NULL: selected selection-block ids (global over the batch, ascending,
 *            -1 padded when the item has fewer than T blocks): Algorithm 1's I
 *   out_branch dev [3,N,Hq,d] or NULL: the three branch outputs before gating
 *   lse, topk_idx and out_branch are optional for inference; ssa_backward needs all three.
 * Errors: NULL, BAD_SHAPE, BAD_HEADS, UNSUPPORTED, MISMATCH, WORKSPACE, HIP.
 */
int ssa_forward(const ssa_params_t *params, const ssa_blocks_t *blocks, const void *q, const void *k,
                const void *v, const void *gates, void *out, float *lse, int32_t *topk_idx, void *out_branch,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * SSA backward: gradients of sum(dout * out) w.r.t. q, k, v, gates, with the selected index sets held
 * constant (no gradient flows through the selection scores or the top-k).  The paper states no backward;
 * this is the softmax-attention gradient of eq. (2)-(4) and of the mean pool of eq. (5).
 *   q,k,v,gates as in ssa_forward; out_branch, lse, topk_idx: what ssa_forward wrote for the same inputs.  A caller
 *   that supplies its own topk_idx (Algorithm 1 takes I as an input) must keep ssa_forward's row format: distinct
 *   selection-block ids of the token's own batch item, the -1 padding at the end of the row; the order of the ids does
 *   not matter.  Rows that break this are not detected: ids out of range, duplicates and -1 in the middle of a row
 *   give undefined gradient values (no memory outside the outputs and the workspace is touched).
 *   dout   dev [N,Hq,d]
 *   dq     dev [N,Hq,d]   dk, dv dev [N,Hkv,d]   dgates dev [N,Hq,3]   all overwritten
 * Errors: as ssa_forward.
 */
int ssa_backward(const ssa_params_t *params, const ssa_blocks_t *blocks, const void *q, const void *k,
                 const void *v, const void *gates, const void *out_branch, const float *lse,
                 const int32_t *topk_idx, const void *dout, void *dq, void *dk, void *dv, void *dgates,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * The top-k decision alone (paper: "The top-k selection blocks with the highest s_slc scores are selected"),
 * on caller-supplied scores: row (t,g) of `scores` (dev float [N,Hkv,S_max]) holds in column j the score of
 * the j-th selection block of t's batch item; columns past the item's block count are ignored.  Writes
 * topk_idx (dev int32 [N,Hkv,T]) exactly as ssa_forward does: the T largest, ties to the lowest block id,
 * ascending ids, -1 padded.  Only n_tokens, n_heads_kv and topk of params are read.
 */
int ssa_topk_from_scores(const ssa_params_t *params, const ssa_blocks_t *blocks, const float *scores,
                         int32_t *topk_idx, void *stream);

/*
 * Learned sparse 3D compression module (Sec. "Sparse 3D Compression", eq. (5)): block-level tokens
 * x_cmp = delta(x + PE(x)), delta = sparse 3D convolution followed by sparse 3D mean pooling, for one tensor x
 * (the keys or the values).  The paper names the three operations only; this library fixes: PE is a table with one
 * row per place inside an m_cmp^3 block, row ((x mod m)*m + (y mod m))*m + (z mod m); the convolution is a
 * submanifold 3x3x3 one over the sparse volume of the token's batch item (outputs at active sites, inactive
 * neighbours contribute nothing) with C = Hkv*d input and output channels and a bias; the mean is over the active
 * tokens of the compression block.  Coordinates must be distinct inside a batch item (otherwise the neighbourhood
 * of a site is not defined; no error is raised).  bf16 only; C in {32, 64, 128, 256}; m_cmp^3 * C <= 16384.
 */
typedef struct {
  const void *pe;   /* dev [m_cmp^3, C]  positional table, dtype of params                                   */
  const void *w;    /* dev [27, C, C]    w[o][c_in][c_out]; o = ((dx+1)*3 + (dy+1))*3 + (dz+1) multiplies the
                                          token at coords + (dx,dy,dz)                                        */
  const void *bias; /* dev [C]                                                                                */
} ssa_cmp_weights_t;

/* Bytes of device workspace of ssa_compress_forward (for_backward == 0) / ssa_compress_backward; 0 on bad input. */
size_t ssa_compress_workspace_bytes(const ssa_params_t *params, const ssa_blocks_t *blocks, int for_backward);

/*
 * Forward of the module.  x dev [N,Hkv,d] (caller token order); x_cmp dev [N_c,Hkv,d], written, row c = compression
 * block c of the handle (ascending (item, Morton) order, the order of ssa_blocks_export(CMP_START)).
 * Asynchronous on `stream`; allocates nothing.  Errors: NULL, MISMATCH, BAD_HEADS, UNSUPPORTED, WORKSPACE, HIP.
 */
int ssa_compress_forward(const ssa_params_t *params, const ssa_blocks_t *blocks, const void *x,
                         const ssa_cmp_weights_t *weights, void *x_cmp, void *workspace, size_t workspace_bytes,
                         void *stream);

/*
 * Backward of the module (chain rule of the three operations; the paper states none).
 *   dx_cmp   dev float [N_c,Hkv,d]  gradient w.r.t. x_cmp (what ssa_backward_pooled writes)
 *   dx_accum dev [N,Hkv,d]          in/out: the gradient w.r.t. x is ADDED to it (it usually already holds the
 *                                   attention's own dk or dv)
 *   dpe dev float [m_cmp^3, C], dw dev float [27, C, C], dbias dev float [C]: overwritten (zeros when N = 0)
 */
int ssa_compress_backward(const ssa_params_t *params, const ssa_blocks_t *blocks, const void *x,
                          const ssa_cmp_weights_t *weights, const float *dx_cmp, void *dx_accum, float *dpe,
                          float *dw, float *dbias, void *workspace, size_t workspace_bytes, void *stream);

/*
 * ssa_forward / ssa_backward with the block-level keys and values supplied by the caller (k_cmp, v_cmp dev
 * [N_c,Hkv,d], e.g. from ssa_compress_forward) instead of the plain mean pool.  ssa_backward_pooled writes the
 * gradients w.r.t. them (dk_cmp, dv_cmp dev float [N_c,Hkv,d]); its dk, dv then hold the selection and window
 * branches only.  Workspace as ssa_workspace_bytes.  bf16 problems the matrix-core kernels cover only
 * (head_dim 32/64/128; backward: 8 or 16 query heads per KV head), otherwise UNSUPPORTED.
 */
int ssa_forward_pooled(const ssa_params_t *params, const ssa_blocks_t *blocks, const void *q, const void *k,
                       const void *v, const void *gates, const void *k_cmp, const void *v_cmp, void *out, float *lse,
                       int32_t *topk_idx, void *out_branch, void *workspace, size_t workspace_bytes, void *stream);
int ssa_backward_pooled(const ssa_params_t *params, const ssa_blocks_t *blocks, const void *q, const void *k,
                        const void *v, const void *gates, const void *k_cmp, const void *v_cmp,
                        const void *out_branch, const float *lse, const int32_t *topk_idx, const void *dout, void *dq,
                        void *dk, void *dv, void *dgates, float *dk_cmp, float *dv_cmp, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * Linear projections of the attention layer around SSA (the query / key / value / output projections of a DiT block
 * with hidden dimension 1024, paper Sec. "Implementation Details"; the paper prints no formula): y = x w^T + bias.
 *   x dev bf16 [N,d_in]; w dev bf16 [d_out,d_in] (one row per output feature); bias dev bf16 [d_out] or NULL;
 *   y dev bf16 [N,d_out].  Backward: dy dev bf16 [N,d_out]; dx dev bf16 [N,d_in] is overwritten (NULL: not computed);
 *   dw dev float [d_out,d_in] and dbias dev float [d_out] (NULL: not computed) are overwritten.
 * bf16 only, fp32 accumulation; d_in and d_out multiples of 128, at most 16384; otherwise UNSUPPORTED.  Forward needs
 * no workspace; backward needs ssa_linear_workspace_bytes(..., 1) bytes.  Asynchronous on `stream`, allocates nothing.
 * Errors: NULL, BAD_SHAPE, UNSUPPORTED, WORKSPACE, HIP.
 */
size_t ssa_linear_workspace_bytes(int32_t n_tokens, int32_t d_in, int32_t d_out, int for_backward);
int ssa_linear_forward(int32_t n_tokens, int32_t d_in, int32_t d_out, const void *x, const void *w, const void *bias,
                       void *y, void *stream);
int ssa_linear_backward(int32_t n_tokens, int32_t d_in, int32_t d_out, const void *x, const void *w, const void *dy,
                        void *dx, float *dw, float *dbias, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Gate predictor (text after eq. (4): the gating score of each module is a linear layer followed by a sigmoid on the
 * input features): gates = sigmoid(x w + bias), one linear layer d_model -> 3*Hq.
 *   x dev [N,d_model]; w dev [d_model, 3*Hq]; bias dev [3*Hq]; gates dev [N,Hq,3] (order cmp, slc, win), the
 *   tensor ssa_forward takes.  Backward: dgates dev [N,Hq,3] (what ssa_backward writes); the gradient w.r.t. x is
 *   ADDED to dx_accum dev [N,d_model] (in/out); dw dev float [d_model, 3*Hq] and dbias dev float [3*Hq] are
 *   overwritten (with zeros when there are no tokens).  Only n_tokens, n_heads_q and dtype of params are read.
 * bf16 only; 3*Hq <= 64; d_model a multiple of 128, at most 16384; otherwise UNSUPPORTED.  Asynchronous on `stream`,
 * allocates nothing.  Errors: NULL, BAD_SHAPE, BAD_HEADS, UNSUPPORTED, WORKSPACE, HIP.
 */
size_t ssa_gate_workspace_bytes(const ssa_params_t *params, int32_t d_model, int for_backward);
int ssa_gate_forward(const ssa_params_t *params, int32_t d_model, const void *x, const void *w, const void *bias,
                     void *gates, void *workspace, size_t workspace_bytes, void *stream);
int ssa_gate_backward(const ssa_params_t *params, int32_t d_model, const void *x, const void *w, const void *gates,
                      const void *dgates, void *dx_accum, float *dw, float *dbias, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * ssa_gate_forward for callers that cannot allocate device memory and have no workspace to hand in: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as ssa_gate_forward, bit for bit;
 * the transposed copy of w (the only scratch memory of the forward pass) lives in a 512 KiB array inside the library
 * instead, one per GPU, held until the process ends.  Limit: d_model <= 4096 (larger: SSA_ERR_UNSUPPORTED; the other
 * limits are those of ssa_gate_forward).  Calls no hipMalloc / hipFree and nothing else that allocates; the first call
 * on a device looks up the array's address (make that call outside a graph capture).  All calls on one GPU share the
 * array, which is rewritten by every call: calls that overlap in time on the same GPU (different streams or threads)
 * race and must be serialised by the caller.  Errors: NULL, BAD_SHAPE, BAD_HEADS, UNSUPPORTED, ALIGNMENT, HIP.
 */
int ssa_gate_forward_static(const ssa_params_t *params, int32_t d_model, const void *x, const void *w, const void *bias,
                            void *gates, void *stream);

/*
 * One full SSA attention layer, composed from the entry points above (the paper gives the parts: projections of the
 * input features to queries, keys and values, gates = sigmoid of a linear layer on the same features, eq. (4), and an
 * output projection; hidden dimension 1024 in its DiT):
 *     q = x wq^T (+bq), k = x wk^T (+bk), v = x wv^T (+bv), gates = sigmoid(x wg + bg),
 *     o = ssa_forward(q, k, v, gates), y = o wo^T (+bo).
 *   x, y, dy, dx  dev bf16 [N, d_model]
 *   weights       host struct of dev bf16 pointers: wq [Hq*d, d_model]; wk, wv [Hkv*d, d_model]; wg [d_model, 3*Hq] and
 *                 bg [3*Hq] (the layout of ssa_gate_forward); wo [d_model, Hq*d]; bq, bk, bv, bo optional (NULL: none).
 *                 pe_k, wc_k, bc_k and pe_v, wc_v, bc_v (the pe, w, bias of ssa_cmp_weights_t for the keys and for the
 *                 values): all six NULL, and the compression branch attends to mean-pooled keys and values; all six
 *                 given, and to the learned module's block tokens (ssa_compress_forward on k and on v, then
 *                 ssa_forward_pooled; backward recomputes them); anything else is SSA_ERR_NULL
 *   saved         dev, ssa_layer_saved_bytes() bytes: the activations forward keeps for backward (q, k, v, gates, o,
 *                 out_branch, lse, topk_idx: their byte offsets from the 256-byte aligned start of the buffer are
 *                 returned in `offsets`, 8 entries in that order, when it is not NULL)
 *   grads         host struct of dev float pointers with the shapes of the weights; dbq, dbk, dbv, dbo optional; the
 *                 six of the compression module required exactly when its weights are given; all overwritten
 * bf16 only; d_model, Hq*d and Hkv*d multiples of 128; 3*Hq <= 64; with the module also its own limits.  Asynchronous on
 * `stream`, allocates nothing.
 * Errors: those of the parts (NULL, BAD_SHAPE, BAD_HEADS, UNSUPPORTED, MISMATCH, WORKSPACE, HIP).
 */
typedef struct {
  const void *wq, *wk, *wv, *wg, *bg, *wo;
  const void *bq, *bk, *bv, *bo;
  const void *pe_k, *wc_k, *bc_k, *pe_v, *wc_v, *bc_v;
} ssa_layer_weights_t;
typedef struct {
  float *dwq, *dwk, *dwv, *dwg, *dbg, *dwo;
  float *dbq, *dbk, *dbv, *dbo;
  float *dpe_k, *dwc_k, *dbc_k, *dpe_v, *dwc_v, *dbc_v;
} ssa_layer_grads_t;
size_t ssa_layer_saved_bytes(const ssa_params_t *params, size_t *offsets);
size_t ssa_layer_workspace_bytes(const ssa_params_t *params, const ssa_blocks_t *blocks, int32_t d_model, int for_backward);
int ssa_layer_forward(const ssa_params_t *params, const ssa_blocks_t *blocks, int32_t d_model, const void *x,
                      const ssa_layer_weights_t *weights, void *y, void *saved, size_t saved_bytes, void *workspace,
                      size_t workspace_bytes, void *stream);
int ssa_layer_backward(const ssa_params_t *params, const ssa_blocks_t *blocks, int32_t d_model, const void *x,
                       const ssa_layer_weights_t *weights, const void *saved, const void *dy, void *dx,
                       const ssa_layer_grads_t *grads, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement hook (not an operation of the paper; for benchmarks that need the duration of single kernels).
 * While enabled, every kernel the library launches is bracketed by a HIP event pair recorded on the launch
 * stream.  ssa_profile_enable(on) clears the totals; ssa_profile_get(i, ...) waits for the recorded events and
 * returns kernel i's name (static string), total milliseconds and number of launches since the last enable.
 * Not thread-safe.
 */
int ssa_profile_enable(int on);
int ssa_profile_num_kernels(void);
int ssa_profile_get(int i, const char **name, double *total_ms, int64_t *launches);

/* Static description of a status code. */
const char *ssa_error_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SSA_H_ */
