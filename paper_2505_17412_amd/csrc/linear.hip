// Linear projections around SSA for gfx950: y = x W^T + b, forward and backward (the query / key / value / output
// projections of an attention layer with hidden dimension 1024, paper Sec. "Implementation Details"; the attention of
// eq. (2)-(4) consumes and produces their tensors).  bf16 in, fp32 accumulation on the matrix cores, bf16 out;
// parameter gradients fp32.
//
//   forward   Y^T tiles: a workgroup owns 128 output features x 128 tokens, the contraction runs in chunks of 64 through
//             LDS (weights and tokens both have the contraction index contiguous, so both operands are plain row
//             reads); output features are the MFMA rows, so a lane ends up with 8 consecutive features of one token and
//             stores 16 bytes.
//   dx        the same kernel on a transposed copy of the weights (dx = dy W).
//   dW        dy^T x contracts over tokens: 32-token tiles of dy and x go through LDS row-major and both operands are
//             transposing LDS reads; the token range is split over workgroups and the fp32 partial tiles are added in a
//             fixed order.  db = column sums of dy in two steps (per 64-token chunk, then over the chunks), fixed order.
// No floating point atomics anywhere.
#include "mfma_common.h"
#include "linear_internal.h"
#include "mfma_qc.h"
#include "profile.h"

namespace {

constexpr int LIN_KC = 64;  // contraction chunk of the forward kernel

struct LinSrc {
  const bf16_t *X[3], *W[3];  // X_i [M][K_i], W_i [O][K_i]
  int K[3];
};

// Y[t][o] = sum_k X[t][k] W[o][k] (+ bias[o]);  X [M][K], W [O][K], Y [M][O];  K % 128 == 0, O % 128 == 0.
// WF x WT wavefronts, each owning CF x CT matrix-instruction tiles (16 features x 16 tokens): the workgroup tile is
// BF = 16*CF*WF features x BT = 16*CT*WT tokens.  Workgroups are dealt round-robin to the 8 XCDs: all feature tiles of
// one token tile run on the same XCD, one after the other, so the token tile is fetched into that XCD's L2 once and the
// weights (a few MB) stay resident in all of them.
// The contraction may run over up to three (X, W) pairs one after the other (Y = sum_i X_i W_i^T): the data gradient
// of projections that share their input is one launch.
template <int WF, int WT, int CF, int CT>
__global__ __launch_bounds__(64 * WF * WT) void lin_nt(LinSrc src, const bf16_t *__restrict__ bias, int M, int O,
                                                       bf16_t *__restrict__ Y) {
  using G = TileGeom<LIN_KC>;
  constexpr int BF = 16 * CF * WF, BT = 16 * CT * WT, NTHR = 64 * WF * WT;
  constexpr int STAGE_W = BF * LIN_KC, STAGE_X = BT * LIN_KC;  // elements per stage
  constexpr int IW = BF * 8 / NTHR, IX = BT * 8 / NTHR;         // 16-byte items per thread and chunk
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t *sw = (bf16_t *)smem, *sx = sw + 2 * STAGE_W;
  const int n_ot = O / BF, n_tt = (M + BT - 1) / BT;
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
  const int tt = (idx / n_ot) * 8 + xcd, ot = idx % n_ot;
  if (tt >= n_tt) return;
  const int m0 = tt * BT, o0 = ot * BF;
  const int tid = threadIdx.x, wid = tid >> 6, lane = tid & 63, n = lane & 15, quad = lane >> 4;
  const int wc = wid % WF, wt = wid / WF;  // the wavefront's features and tokens inside the tile
  f32x4 acc[CF][CT];
#pragma unroll
  for (int ci = 0; ci < CF; ++ci)
#pragma unroll
    for (int ti = 0; ti < CT; ++ti) acc[ci][ti] = f32x4{0.f, 0.f, 0.f, 0.f};
  // Two chunks are in flight in registers (A: the next chunk, B: the one after), so a global load has two loop trips
  // to arrive; the loop is unrolled by two to alternate the register sets.
  bf16x8 rwA[IW], rxA[IX], rwB[IW], rxB[IX];
  const int K = src.K[0] + src.K[1] + src.K[2];  // unused pairs have K = 0
  auto fetch = [&](int kf, bf16x8 (&rw)[IW], bf16x8 (&rx)[IX]) {
    // which pair the flat contraction index kf falls into (every K_i is a multiple of 128, so a chunk never straddles)
    const int p = kf < src.K[0] ? 0 : (kf < src.K[0] + src.K[1] ? 1 : 2);
    const int k0 = kf - (p > 0 ? src.K[0] : 0) - (p > 1 ? src.K[1] : 0), Kp = src.K[p];
    const bf16_t *X = src.X[p], *W = src.W[p];
#pragma unroll
    for (int i = 0; i < IW; ++i) {
      const int it = tid + NTHR * i, row = it >> 3, seg = it & 7;
      rw[i] = ld8(W + (size_t)(o0 + row) * Kp + k0 + 8 * seg);
    }
#pragma unroll
    for (int i = 0; i < IX; ++i) {
      const int it = tid + NTHR * i, row = it >> 3, seg = it & 7, t = m0 + row;
      rx[i] = t < M ? ld8(X + (size_t)t * Kp + k0 + 8 * seg) : zero8();
    }
  };
  auto stash = [&](int buf, const bf16x8 (&rw)[IW], const bf16x8 (&rx)[IX]) {
#pragma unroll
    for (int i = 0; i < IW; ++i) {
      const int it = tid + NTHR * i, row = it >> 3, seg = it & 7;
      *reinterpret_cast<bf16x8 *>(sw + buf * STAGE_W + (row >> 5) * G::ROW_ELEMS + G::row_off(row & 31, seg)) = rw[i];
    }
#pragma unroll
    for (int i = 0; i < IX; ++i) {
      const int it = tid + NTHR * i, row = it >> 3, seg = it & 7;
      *reinterpret_cast<bf16x8 *>(sx + buf * STAGE_X + (row >> 5) * G::ROW_ELEMS + G::row_off(row & 31, seg)) = rx[i];
    }
  };
  auto compute = [&](int buf) {
    const bf16_t *cw = sw + buf * STAGE_W + (CF / 2) * wc * G::ROW_ELEMS, *cx = sx + buf * STAGE_X + (CT / 2) * wt * G::ROW_ELEMS;
#pragma unroll
    for (int ks = 0; ks < LIN_KC / 32; ++ks) {
      bf16x8 a[CF], b[CT];
#pragma unroll
      for (int ci = 0; ci < CF; ++ci) a[ci] = lds_row_operand<LIN_KC>(cw + (ci >> 1) * G::ROW_ELEMS, ci & 1, ks);
#pragma unroll
      for (int ti = 0; ti < CT; ++ti) b[ti] = lds_row_operand<LIN_KC>(cx + (ti >> 1) * G::ROW_ELEMS, ti & 1, ks);
#pragma unroll
      for (int ci = 0; ci < CF; ++ci)
#pragma unroll
        for (int ti = 0; ti < CT; ++ti) acc[ci][ti] = mfma16(a[ci], b[ti], acc[ci][ti]);
    }
  };
  // K is a multiple of 128: an even number of chunks
  fetch(0, rwA, rxA);
  fetch(LIN_KC, rwB, rxB);
  stash(0, rwA, rxA);
  __syncthreads();
  for (int k0 = 0; k0 < K; k0 += 2 * LIN_KC) {
    // stage 0 holds chunk k0, registers B chunk k0 + 64
    if (k0 + 2 * LIN_KC < K) fetch(k0 + 2 * LIN_KC, rwA, rxA);
    compute(0);
    stash(1, rwB, rxB);  // stage 1 was last read before the previous barrier
    __syncthreads();
    if (k0 + 3 * LIN_KC < K) fetch(k0 + 3 * LIN_KC, rwB, rxB);
    compute(1);
    if (k0 + 2 * LIN_KC < K) stash(0, rwA, rxA);
    __syncthreads();
  }
  // MFMA row r of sub-tile a of a 32-row tile is row 8*(r >> 2) + 4*a + (r & 3): with r = 4*quad + i the two sub-tiles
  // of a feature tile give the lane features 8*quad .. 8*quad+7; column n of token sub-tile b is token row
  // 8*(n >> 2) + 4*b + (n & 3).
#pragma unroll
  for (int cr = 0; cr < CF / 2; ++cr) {
    const int ch = o0 + 16 * CF * wc + 32 * cr + 8 * quad;
    float bs[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) bs[j] = bias ? bf16_to_f32(bias[ch + j]) : 0.f;
#pragma unroll
    for (int ti = 0; ti < CT; ++ti) {
      const int t = m0 + 16 * CT * wt + 32 * (ti >> 1) + 8 * (n >> 2) + 4 * (ti & 1) + (n & 3);
      if (t >= M) continue;
      bf16x8 o;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        o[i] = (__bf16)(acc[2 * cr][ti][i] + bs[i]);
        o[4 + i] = (__bf16)(acc[2 * cr + 1][ti][i] + bs[4 + i]);
      }
      *reinterpret_cast<bf16x8 *>(Y + (size_t)t * O + ch) = o;
    }
  }
}

// Wt[k][o] = W[o][k]: 32 x 32 tiles through LDS, both sides coalesced.
__global__ __launch_bounds__(256) void lin_transpose(const bf16_t *__restrict__ W, int O, int K, bf16_t *__restrict__ Wt) {
  __shared__ bf16_t t[32][33];
  const int k0 = blockIdx.x * 32, o0 = blockIdx.y * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
  for (int r = ty; r < 32; r += 8) t[r][tx] = W[(size_t)(o0 + r) * K + k0 + tx];
  __syncthreads();
#pragma unroll
  for (int r = ty; r < 32; r += 8) Wt[(size_t)(k0 + r) * O + o0 + tx] = t[tx][r];
}

// part[split][o][k] = sum over the split's tokens of dY[t][o] X[t][k]: workgroup = 128 x 128 output tile, one split.
__global__ __launch_bounds__(256) void lin_tn(const bf16_t *__restrict__ dY, const bf16_t *__restrict__ X, int M, int O,
                                              int K, int tok_per_split, float *__restrict__ part) {
  using G = TileGeom<128>;
  __shared__ __align__(16) bf16_t sy[2][G::ROW_ELEMS], sx[2][G::ROW_ELEMS];
  const int n_kt = K / 128;
  const int ot = blockIdx.x / n_kt, kt = blockIdx.x % n_kt, split = blockIdx.y;
  const int o0 = ot * 128, c0 = kt * 128;
  const int t_begin = split * tok_per_split, t_end = min(M, t_begin + tok_per_split);
  const int tid = threadIdx.x, wid = tid >> 6, lane = tid & 63, n = lane & 15, quad = lane >> 4;
  const int wo = wid & 1, wk = wid >> 1;
  f32x4 acc[4][4];
#pragma unroll
  for (int oi = 0; oi < 4; ++oi)
#pragma unroll
    for (int ki = 0; ki < 4; ++ki) acc[oi][ki] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 ry[2], rx[2];
  auto fetch = [&](int t0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int it = tid + 256 * i, row = it >> 4, seg = it & 15, t = t0 + row;
      ry[i] = t < t_end ? ld8(dY + (size_t)t * O + o0 + 8 * seg) : zero8();
      rx[i] = t < t_end ? ld8(X + (size_t)t * K + c0 + 8 * seg) : zero8();
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int it = tid + 256 * i, row = it >> 4, seg = it & 15;
      *reinterpret_cast<bf16x8 *>(&sy[buf][G::row_off(row, seg)]) = ry[i];
      *reinterpret_cast<bf16x8 *>(&sx[buf][G::row_off(row, seg)]) = rx[i];
    }
  };
  if (t_begin < t_end) {
    fetch(t_begin);
    stash(0);
  }
  __syncthreads();
  for (int t0 = t_begin, buf = 0; t0 < t_end; t0 += 32, buf ^= 1) {
    const bool more = t0 + 32 < t_end;
    if (more) fetch(t0 + 32);
    bf16x8 a[4], b[4];
#pragma unroll
    for (int oi = 0; oi < 4; ++oi) a[oi] = lds_tr_operand<128>(sy[buf], 4 * wo + oi);
#pragma unroll
    for (int ki = 0; ki < 4; ++ki) b[ki] = lds_tr_operand<128>(sx[buf], 4 * wk + ki);
#pragma unroll
    for (int oi = 0; oi < 4; ++oi)
#pragma unroll
      for (int ki = 0; ki < 4; ++ki) acc[oi][ki] = mfma16(a[oi], b[ki], acc[oi][ki]);
    if (more) stash(buf ^ 1);
    __syncthreads();
  }
  float *dst = part + (size_t)split * O * K;
#pragma unroll
  for (int oi = 0; oi < 4; ++oi)
#pragma unroll
    for (int ki = 0; ki < 4; ++ki)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        dst[(size_t)(o0 + 64 * wo + 16 * oi + 4 * quad + i) * K + c0 + 64 * wk + 16 * ki + n] = acc[oi][ki][i];
}

// out[j] = sum_s part[s][j], s ascending
__global__ void lin_sum_parts(const float *__restrict__ part, int n_parts, size_t len, float *__restrict__ out) {
  const size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= len) return;
  float s = 0.f;
  for (int p = 0; p < n_parts; ++p) s += part[(size_t)p * len + j];
  out[j] = s;
}

// Column sums of dY (the bias gradient) in two steps, both with a fixed order of additions.
// Step 1: part[chunk][o] = sum of dY[t][o] over the chunk's COLSUM_CHUNK tokens; a thread owns 8 columns and every
// `phases`-th token, the phases are added in order through LDS.  O % 8 == 0, O / 8 <= 256 or a multiple of 256.
constexpr int COLSUM_CHUNK = 64;
__global__ __launch_bounds__(256) void lin_colsum(const bf16_t *__restrict__ dY, int M, int O, float *__restrict__ part) {
  __shared__ float red[2048];
  const int cols8 = O / 8;
  const int phases = cols8 >= 256 ? 1 : 256 / cols8;
  const int t_begin = blockIdx.x * COLSUM_CHUNK, t_end = min(M, t_begin + COLSUM_CHUNK);
  for (int cg0 = 0; cg0 < cols8; cg0 += 256) {
    const int ph = threadIdx.x / cols8, cg = cg0 + threadIdx.x % cols8;
    const bool active = ph < phases && cg < cols8;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (active) {
#pragma unroll 4
      for (int t = t_begin + ph; t < t_end; t += phases) {
        const bf16x8 v = ld8(dY + (size_t)t * O + 8 * cg);
#pragma unroll
        for (int j = 0; j < 8; ++j) s[j] += (float)v[j];
      }
    }
    for (int g = 0; g < phases; ++g) {
      __syncthreads();
      if (active && ph == g)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int c = 8 * (cg - cg0) + j;
          red[c] = g == 0 ? s[j] : red[c] + s[j];
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < 8 * min(256, cols8 - cg0); c += 256) part[(size_t)blockIdx.x * O + 8 * cg0 + c] = red[c];
    __syncthreads();
  }
}
// Step 2: out[o] = sum over the parts; a workgroup owns 8 columns, 32 thread rows each add every 32nd part, then the
// rows are added in order.
__global__ __launch_bounds__(256) void lin_colsum_finish(const float *__restrict__ part, int n_parts, int O, float *__restrict__ out) {
  __shared__ float red[32][8];
  const int col = blockIdx.x * 8 + (threadIdx.x & 7), row = threadIdx.x >> 3;
  float s = 0.f;
  if (col < O)
    for (int p = row; p < n_parts; p += 32) s += part[(size_t)p * O + col];
  red[row][threadIdx.x & 7] = s;
  __syncthreads();
  if (row == 0 && col < O) {
    float t = 0.f;
#pragma unroll
    for (int r = 0; r < 32; ++r) t += red[r][threadIdx.x & 7];
    out[col] = t;
  }
}

struct LinPlan {
  int splits, tok_per_split, bias_parts;
  size_t wt, part, bpart, total;
};

LinPlan lin_plan(int M, int d_in, int d_out) {
  LinPlan p{};
  const int tiles = (d_out / 128) * (d_in / 128);
  // three workgroups per compute unit; two for skinny outputs, where the traffic of the partial tiles weighs more
  int s = ((tiles >= 16 ? 768 : 512) + tiles - 1) / tiles;
  const int max_s = (M + 255) / 256;   // at least 256 tokens per split
  if (s > max_s) s = max_s;
  if (s < 1) s = 1;
  p.tok_per_split = (((M + s - 1) / s) + 31) / 32 * 32;
  if (p.tok_per_split < 32) p.tok_per_split = 32;
  p.splits = M > 0 ? (M + p.tok_per_split - 1) / p.tok_per_split : 1;
  size_t off = 0;
  p.wt = off; off += align_up((size_t)d_in * d_out * sizeof(bf16_t), 256);
  p.part = off; off += align_up((size_t)p.splits * d_in * d_out * sizeof(float), 256);
  p.bias_parts = M > 0 ? (M + COLSUM_CHUNK - 1) / COLSUM_CHUNK : 1;
  p.bpart = off; off += align_up((size_t)p.bias_parts * d_out * sizeof(float), 256);
  p.total = off;
  return p;
}


}  // namespace

int lin_nt_multi(int n_src, const void *const *X, const void *const *W, const int *K, const void *bias, int M, int O,
                 void *Y, hipStream_t s) {
  constexpr int WF = 2, WT = 2, CF = 4, CT = 4, BF = 16 * CF * WF, BT = 16 * CT * WT;
  const size_t lds = (size_t)2 * (BF + BT) * LIN_KC * sizeof(bf16_t);  // two stages of weights and tokens
  static const hipError_t attr =
      hipFuncSetAttribute((const void *)lin_nt<WF, WT, CF, CT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (attr != hipSuccess) return SSA_ERR_HIP;
  LinSrc src{};
  for (int i = 0; i < 3; ++i) {
    src.X[i] = i < n_src ? (const bf16_t *)X[i] : nullptr;
    src.W[i] = i < n_src ? (const bf16_t *)W[i] : nullptr;
    src.K[i] = i < n_src ? K[i] : 0;
  }
  const int n_ot = O / BF, n_tt = (M + BT - 1) / BT;
  const unsigned grid = (unsigned)(8 * ((n_tt + 7) / 8) * n_ot);
  lin_nt<WF, WT, CF, CT><<<grid, 64 * WF * WT, lds, s>>>(src, (const bf16_t *)bias, M, O, (bf16_t *)Y);
  return SSA_OK;
}

void lin_transpose_w(const void *w, int d_out, int d_in, void *wt, hipStream_t s) {
  lin_transpose<<<dim3(d_in / 32, d_out / 32), 256, 0, s>>>((const bf16_t *)w, d_out, d_in, (bf16_t *)wt);
}

size_t lin_dw_workspace(int M, int d_in, int d_out) {
  const LinPlan p = lin_plan(M, d_in, d_out);
  return p.total - p.part;
}

// dw [d_out][d_in] = dy^T x, dbias (optional) = column sums of dy; ws holds lin_dw_workspace() bytes, 256-byte aligned
int lin_dw(int M, int d_in, int d_out, const void *x, const void *dy, float *dw, float *dbias, void *ws, hipStream_t s) {
  const LinPlan pl = lin_plan(M, d_in, d_out);
  float *part = (float *)ws, *bpart = (float *)((char *)ws + (pl.bpart - pl.part));
  lin_tn<<<dim3((d_out / 128) * (d_in / 128), pl.splits), 256, 0, s>>>((const bf16_t *)dy, (const bf16_t *)x, M, d_out, d_in,
                                                                     pl.tok_per_split, part);
  const size_t len = (size_t)d_in * d_out;
  lin_sum_parts<<<(unsigned)((len + 255) / 256), 256, 0, s>>>(part, pl.splits, len, dw);
  if (dbias) {
    lin_colsum<<<pl.bias_parts, 256, 0, s>>>((const bf16_t *)dy, M, d_out, bpart);
    lin_colsum_finish<<<(d_out + 7) / 8, 256, 0, s>>>(bpart, pl.bias_parts, d_out, dbias);
  }
  return SSA_OK;
}

int lin_check(int n_tokens, int d_in, int d_out) {
  if (n_tokens < 0) return SSA_ERR_BAD_SHAPE;
  if (d_in < 128 || d_out < 128 || d_in % 128 != 0 || d_out % 128 != 0 || d_in > 16384 || d_out > 16384) return SSA_ERR_UNSUPPORTED;
  if ((long long)n_tokens * (d_in > d_out ? d_in : d_out) >= (1ll << 31)) return SSA_ERR_BAD_SHAPE;
  return SSA_OK;
}

extern "C" size_t ssa_linear_workspace_bytes(int32_t n_tokens, int32_t d_in, int32_t d_out, int for_backward) {
  if (lin_check(n_tokens, d_in, d_out) != SSA_OK) return 0;
  return for_backward ? lin_plan(n_tokens, d_in, d_out).total + 256 : 256;
}

extern "C" int ssa_linear_forward(int32_t n_tokens, int32_t d_in, int32_t d_out, const void *x, const void *w,
                                  const void *bias, void *y, void *stream) {
  const int rc = lin_check(n_tokens, d_in, d_out);
  if (rc != SSA_OK) return rc;
  if (n_tokens == 0) return SSA_OK;
  if (!x || !w || !y) return SSA_ERR_NULL;
  if (!aligned16(x, w, bias, y)) return SSA_ERR_ALIGNMENT;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(PROF_LINEAR_FWD, s);
  const int lrc = lin_nt_multi(1, &x, &w, &d_in, bias, n_tokens, d_out, y, s);
  if (lrc != SSA_OK) return lrc;
  SSA_HIP_TRY(hipGetLastError());
  return SSA_OK;
}

extern "C" int ssa_linear_backward(int32_t n_tokens, int32_t d_in, int32_t d_out, const void *x, const void *w,
                                   const void *dy, void *dx, float *dw, float *dbias, void *ws_, size_t ws_bytes,
                                   void *stream) {
  const int rc = lin_check(n_tokens, d_in, d_out);
  if (rc != SSA_OK) return rc;
  if (!dw) return SSA_ERR_NULL;
  hipStream_t s = (hipStream_t)stream;
  if (n_tokens == 0) {  // no tokens: the parameter gradients are zero
    const size_t len = (size_t)d_in * d_out;  // a sum over zero partials writes zeros
    lin_sum_parts<<<(unsigned)((len + 255) / 256), 256, 0, s>>>(nullptr, 0, len, dw);
    if (dbias) lin_sum_parts<<<(d_out + 255) / 256, 256, 0, s>>>(nullptr, 0, (size_t)d_out, dbias);
    SSA_HIP_TRY(hipGetLastError());
    return SSA_OK;
  }
  if (!x || !w || !dy) return SSA_ERR_NULL;
  if (!aligned16(x, w, dy, dx, dw, dbias)) return SSA_ERR_ALIGNMENT;
  if (!ws_ || ws_bytes < ssa_linear_workspace_bytes(n_tokens, d_in, d_out, 1)) return SSA_ERR_WORKSPACE;
  const LinPlan pl = lin_plan(n_tokens, d_in, d_out);
  char *ws = (char *)align_up((size_t)ws_, 256);
  ProfScope ps(PROF_LINEAR_BWD, s);
  if (dx) {
    const void *wt = ws + pl.wt;
    lin_transpose_w(w, d_out, d_in, ws + pl.wt, s);
    const int lrc = lin_nt_multi(1, &dy, &wt, &d_out, nullptr, n_tokens, d_in, dx, s);
    if (lrc != SSA_OK) return lrc;
  }
  lin_dw(n_tokens, d_in, d_out, x, dy, dw, dbias, ws + pl.part, s);
  SSA_HIP_TRY(hipGetLastError());
  return SSA_OK;
}
