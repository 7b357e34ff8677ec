// Gate predictor of SSA for gfx950: gates = sigmoid(x W + b), forward and backward (paper, text after eq. (4): the
// gating scores come from a linear layer followed by a sigmoid on the input features).
//
// Reading: one linear layer d_model -> J = 3*H_q with bias; output [N][H_q][3] in the branch order (cmp, slc, win).
// The layer is skinny (J <= 64 outputs), so every kernel here is bound by streaming x (or dx) once through HBM;
// the contractions run on the matrix cores only to keep the vector ALU out of the way.
//   forward   a wave owns 16 tokens: A = x rows straight from memory, B = W^T (contraction index contiguous, a
//             small transposed copy), sigmoid in the epilogue;
//   backward  dz = dgates * g * (1 - g) (bf16, padded to 64 columns);  dx += dz W^T with dims as MFMA rows, so a
//             lane holds 4 consecutive dims of one token;  dW = x^T dz contracts over tokens: 32-token tiles of x and
//             dz go through LDS row-major and both operands are transposing LDS reads;  db = column sums of dz.
// No floating point atomics: per-chunk partial sums are added in a fixed order.
#include "mfma_common.h"
#include "mfma_qc.h"
#include "profile.h"

namespace {

constexpr int JP = 64;  // padded gate count (columns of dz and of the padded weights)

// Wt[j][k] = w[k][j] (j < J), zero rows up to 16*ceil(J/16);  Wp[k][j] = w[k][j], zero for J <= j < 64
__global__ void g_prep_w(const bf16_t *__restrict__ w, int Dm, int J, int JR, bf16_t *__restrict__ wt, bf16_t *__restrict__ wp) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (wt && i < (size_t)JR * Dm) {
    const int j = (int)(i / Dm), k = (int)(i % Dm);
    wt[i] = j < J ? w[(size_t)k * J + j] : (bf16_t)0;
  }
  if (wp && i < (size_t)Dm * JP) {
    const int k = (int)(i / JP), j = (int)(i % JP);
    wp[i] = j < J ? w[(size_t)k * J + j] : (bf16_t)0;
  }
}

// gates[tok][j] = sigmoid(sum_k x[tok][k] w[k][j] + b[j]); NB = blocks of 16 gate columns
template <int NB>
__global__ __launch_bounds__(256) void g_fwd(const bf16_t *__restrict__ x, const bf16_t *__restrict__ wt,
                                             const bf16_t *__restrict__ bias, int N, int Dm, int J, bf16_t *__restrict__ gates) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int t0 = (blockIdx.x * 4 + wid) * 16;
  if (t0 >= N) return;
  const int tok = min(t0 + n, N - 1);  // rows past the end repeat the last token and are not stored
  const bf16_t *xr = x + (size_t)tok * Dm + 8 * quad;
  f32x4 acc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int ks = 0; ks < Dm / 32; ++ks) {
    const bf16x8 av = ld8(xr + 32 * ks);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = mfma16(av, ld8(wt + (size_t)(16 * nb + n) * Dm + 32 * ks + 8 * quad), acc[nb]);
  }
  // C layout: lane holds gate column 16*nb + n of tokens t0 + 4*quad + i
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int j = 16 * nb + n;
    if (j >= J) continue;
    const float b = bf16_to_f32(bias[j]);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int t = t0 + 4 * quad + i;
      if (t < N) gates[(size_t)t * J + j] = f32_to_bf16(1.0f / (1.0f + __expf(-(acc[nb][i] + b))));
    }
  }
}

// dz[tok][j] = dgates * g * (1 - g) for j < J, zero up to column 63 (bf16); per-chunk column sums for db
__global__ __launch_bounds__(256) void g_dz(const bf16_t *__restrict__ gates, const bf16_t *__restrict__ dgates, int N, int J,
                                            int chunk, bf16_t *__restrict__ dz, float *__restrict__ pb) {
  __shared__ float col[4][JP];
  const int j = threadIdx.x & 63, r = threadIdx.x >> 6;
  const int b = blockIdx.x * chunk, e = min(N, b + chunk);
  float s = 0.f;
  for (int t = b + r; t < e; t += 4) {  // row lane r visits tokens b+r, b+r+4, ..: a fixed order per (r, j)
    float v = 0.f;
    if (j < J) {
      const float g = bf16_to_f32(gates[(size_t)t * J + j]);
      v = bf16_to_f32(dgates[(size_t)t * J + j]) * g * (1.0f - g);
    }
    dz[(size_t)t * JP + j] = f32_to_bf16(v);
    s += v;
  }
  col[r][j] = s;
  __syncthreads();
  if (r == 0) pb[(size_t)blockIdx.x * JP + j] = (col[0][j] + col[1][j]) + (col[2][j] + col[3][j]);
}

// dx[tok][dim] += sum_j dz[tok][j] w[dim][j]: MFMA rows = dims (A = padded weights), columns = tokens (B = dz rows)
__global__ __launch_bounds__(256) void g_dx(const bf16_t *__restrict__ dz, const bf16_t *__restrict__ wp, int N, int Dm,
                                            bf16_t *dx) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int t0 = (blockIdx.x * 4 + wid) * 16;
  if (t0 >= N) return;
  const int tok = t0 + n;
  const bool ok = tok < N;
  bf16x8 bz[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) bz[ks] = ok ? ld8(dz + (size_t)tok * JP + 32 * ks + 8 * quad) : zero8();
  for (int mb = 0; mb < Dm / 16; ++mb) {
    const bf16_t *wr = wp + (size_t)(16 * mb + n) * JP + 8 * quad;
    f32x4 acc = mfma16(ld8(wr), bz[0], f32x4{0.f, 0.f, 0.f, 0.f});
    acc = mfma16(ld8(wr + 32), bz[1], acc);
    // C layout: lane holds dims 16*mb + 4*quad .. +3 of token column n: 8 contiguous bytes of dx
    if (ok) {
      bf16_t *d = dx + (size_t)tok * Dm + 16 * mb + 4 * quad;
      const bf16x4 cur = *reinterpret_cast<const bf16x4 *>(d);
      bf16x4 r;
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = (__bf16)((float)cur[i] + acc[i]);
      *reinterpret_cast<bf16x4 *>(d) = r;
    }
  }
}

// dW partial: part[chunk][dim][j] = sum over the chunk's tokens of x[tok][dim] dz[tok][j]; a workgroup owns 128 dims
// (wave w the 16-row blocks w and w+4) and all 64 (padded) gate columns.
__global__ __launch_bounds__(256) void g_dw(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dz, int N, int Dm,
                                            int chunk, float *__restrict__ part) {
  using GX = TileGeom<128>;
  using GZ = TileGeom<JP>;
  __shared__ __align__(16) bf16_t sx[GX::ROW_ELEMS], sz[GZ::ROW_ELEMS];
  const int d0 = blockIdx.x * 128, s = blockIdx.y;
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  f32x4 acc[2][JP / 16];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int nb = 0; nb < JP / 16; ++nb) acc[a][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int b = s * chunk, e = min(N, b + chunk);
  for (int t0 = b; t0 < e; t0 += 32) {
    for (int it = threadIdx.x; it < GX::ROW_ITEMS; it += 256) {
      const int row = it / 16, seg = it % 16, t = t0 + row;
      *reinterpret_cast<bf16x8 *>(sx + GX::row_off(row, seg)) = t < e ? ld8(x + (size_t)t * Dm + d0 + 8 * seg) : zero8();
    }
    {
      const int row = threadIdx.x / 8, seg = threadIdx.x % 8, t = t0 + row;  // 32 rows x 8 segments = 256 items
      *reinterpret_cast<bf16x8 *>(sz + GZ::row_off(row, seg)) = t < e ? ld8(dz + (size_t)t * JP + 8 * seg) : zero8();
    }
    __syncthreads();
    bf16x8 av[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) av[a] = lds_tr_operand<128>(sx, wid + 4 * a);
#pragma unroll
    for (int nb = 0; nb < JP / 16; ++nb) {
      const bf16x8 bv = lds_tr_operand<JP>(sz, nb);
#pragma unroll
      for (int a = 0; a < 2; ++a) acc[a][nb] = mfma16(av[a], bv, acc[a][nb]);
    }
    __syncthreads();
  }
  float *dst = part + (size_t)s * Dm * JP;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int nb = 0; nb < JP / 16; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) dst[(size_t)(d0 + 16 * (wid + 4 * a) + 4 * quad + i) * JP + 16 * nb + n] = acc[a][nb][i];
}

// out[r][j] (row stride J, j < J) = sum over parts p = 0 .. n_parts-1 of part[p][r][j] (row stride 64), in order
__global__ void g_sum_parts(const float *__restrict__ part, int n_parts, int rows, int J, float *__restrict__ out) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)rows * J) return;
  const int r = (int)(i / J), j = (int)(i % J);
  float s = 0.f;
  for (int p = 0; p < n_parts; ++p) s += part[((size_t)p * rows + r) * JP + j];
  out[i] = s;
}

struct GatePlan {
  size_t wt, wp, dz, pw, pb, total;
  int chunks, chunk;
};

GatePlan gate_plan(int N, int Dm, int J, bool backward) {
  GatePlan p{};
  size_t off = 0;
  auto take = [&](size_t n) { size_t r = off; off += align_up(n, 256); return r; };
  if (!backward) {
    p.wt = take((size_t)((J + 15) / 16 * 16) * Dm * 2);
  } else {
    p.wp = take((size_t)Dm * JP * 2);
    p.dz = take((size_t)N * JP * 2);
    p.chunks = N > 0 ? (N + 1023) / 1024 : 1;
    if (p.chunks > 64) p.chunks = 64;
    p.chunk = ((N + p.chunks - 1) / p.chunks + 31) / 32 * 32;
    if (p.chunk < 32) p.chunk = 32;
    p.pw = take((size_t)p.chunks * Dm * JP * 4);
    p.pb = take((size_t)p.chunks * JP * 4);
  }
  p.total = off;
  return p;
}

int gate_check(const ssa_params_t *p, int d_model, int *J) {
  if (!p) return SSA_ERR_NULL;
  if (p->n_tokens < 0) return SSA_ERR_BAD_SHAPE;
  if (p->n_heads_q < 1) return SSA_ERR_BAD_HEADS;
  if (p->dtype != SSA_BF16) return SSA_ERR_UNSUPPORTED;
  if (3 * p->n_heads_q > JP || d_model < 128 || d_model % 128 != 0 || d_model > 16384) return SSA_ERR_UNSUPPORTED;
  if ((long long)p->n_tokens * d_model >= (1ll << 40)) return SSA_ERR_BAD_SHAPE;
  *J = 3 * p->n_heads_q;
  return SSA_OK;
}

}  // namespace

extern "C" size_t ssa_gate_workspace_bytes(const ssa_params_t *p, int32_t d_model, int for_backward) {
  int J;
  if (gate_check(p, d_model, &J) != SSA_OK) return 0;
  return gate_plan(p->n_tokens, d_model, J, for_backward != 0).total + 256;
}

extern "C" int ssa_gate_forward(const ssa_params_t *p, int32_t d_model, const void *x, const void *w, const void *bias,
                                void *gates, void *ws_, size_t ws_bytes, void *stream) {
  int J;
  const int rc = gate_check(p, d_model, &J);
  if (rc != SSA_OK) return rc;
  const int N = p->n_tokens;
  if (N == 0) return SSA_OK;
  if (!x || !w || !bias || !gates) return SSA_ERR_NULL;
  if (!ws_ || ws_bytes < ssa_gate_workspace_bytes(p, d_model, 0)) return SSA_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const GatePlan pl = gate_plan(N, d_model, J, false);
  char *ws = (char *)align_up((size_t)ws_, 256);
  bf16_t *wt = (bf16_t *)(ws + pl.wt);
  const int NB = (J + 15) / 16, JR = 16 * NB;
  ProfScope ps(PROF_GATE_FWD, s);
  g_prep_w<<<(unsigned)(((size_t)JR * d_model + 255) / 256), 256, 0, s>>>((const bf16_t *)w, d_model, J, JR, wt, nullptr);
  const unsigned grid = (unsigned)((N + 63) / 64);
  switch (NB) {
    case 1: g_fwd<1><<<grid, 256, 0, s>>>((const bf16_t *)x, wt, (const bf16_t *)bias, N, d_model, J, (bf16_t *)gates); break;
    case 2: g_fwd<2><<<grid, 256, 0, s>>>((const bf16_t *)x, wt, (const bf16_t *)bias, N, d_model, J, (bf16_t *)gates); break;
    case 3: g_fwd<3><<<grid, 256, 0, s>>>((const bf16_t *)x, wt, (const bf16_t *)bias, N, d_model, J, (bf16_t *)gates); break;
    default: g_fwd<4><<<grid, 256, 0, s>>>((const bf16_t *)x, wt, (const bf16_t *)bias, N, d_model, J, (bf16_t *)gates); break;
  }
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

extern "C" int ssa_gate_backward(const ssa_params_t *p, int32_t d_model, const void *x, const void *w, const void *gates,
                                 const void *dgates, void *dx_accum, float *dw, float *dbias, void *ws_, size_t ws_bytes,
                                 void *stream) {
  int J;
  const int rc = gate_check(p, d_model, &J);
  if (rc != SSA_OK) return rc;
  const int N = p->n_tokens;
  if (N == 0) return SSA_OK;
  if (!x || !w || !gates || !dgates || !dx_accum || !dw || !dbias) return SSA_ERR_NULL;
  if (!ws_ || ws_bytes < ssa_gate_workspace_bytes(p, d_model, 1)) return SSA_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const GatePlan pl = gate_plan(N, d_model, J, true);
  char *ws = (char *)align_up((size_t)ws_, 256);
  bf16_t *wp = (bf16_t *)(ws + pl.wp), *dz = (bf16_t *)(ws + pl.dz);
  float *pw = (float *)(ws + pl.pw), *pb = (float *)(ws + pl.pb);
  ProfScope ps(PROF_GATE_BWD, s);
  g_prep_w<<<(unsigned)(((size_t)d_model * JP + 255) / 256), 256, 0, s>>>((const bf16_t *)w, d_model, J, 0, nullptr, wp);
  g_dz<<<pl.chunks, 256, 0, s>>>((const bf16_t *)gates, (const bf16_t *)dgates, N, J, pl.chunk, dz, pb);
  g_sum_parts<<<1, 64, 0, s>>>(pb, pl.chunks, 1, J, dbias);
  g_dx<<<(unsigned)((N + 63) / 64), 256, 0, s>>>(dz, wp, N, d_model, (bf16_t *)dx_accum);
  g_dw<<<dim3(d_model / 128, pl.chunks), 256, 0, s>>>((const bf16_t *)x, dz, N, d_model, pl.chunk, pw);
  g_sum_parts<<<(unsigned)(((size_t)d_model * J + 255) / 256), 256, 0, s>>>(pw, pl.chunks, d_model, J, dw);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}
