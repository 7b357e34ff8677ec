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
//             dz go through LDS row-major and both operands are transposing LDS reads;  db = column sums of dz
//             (one more matrix instruction with an all-ones operand in the same kernel).
// No floating point atomics: per-chunk partial sums are added in a fixed order.
#include "mfma_common.h"
#include "mfma_qc.h"
#include "profile.h"

#include <mutex>

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

// gates[tok][j] = sigmoid(sum_k x[tok][k] w[k][j] + b[j]); NB = blocks of 16 gate columns.  A wave owns two tiles of
// 16 tokens (every weight operand feeds two matrix instructions); four contraction steps are issued per loop trip, so
// eight 1 KB row loads per wave are in flight.
template <int NB>
__global__ __launch_bounds__(256) void g_fwd(const bf16_t *__restrict__ x, const bf16_t *__restrict__ wt,
                                             const bf16_t *__restrict__ bias, int N, int Dm, int J, bf16_t *__restrict__ gates) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int t0 = (blockIdx.x * 4 + wid) * 32;
  if (t0 >= N) return;
  const bf16_t *xr[2];
#pragma unroll
  for (int a = 0; a < 2; ++a) xr[a] = x + (size_t)min(t0 + 16 * a + n, N - 1) * Dm + 8 * quad;  // rows past the end
  f32x4 acc[2][NB];                                                                       // repeat the last token
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[a][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int k4 = 0; k4 < Dm / 128; ++k4) {  // d_model is a multiple of 128: four contraction steps per trip
    bf16x8 av[2][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      av[0][u] = ld8(xr[0] + 128 * k4 + 32 * u);
      av[1][u] = ld8(xr[1] + 128 * k4 + 32 * u);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const bf16x8 bv = ld8(wt + (size_t)(16 * nb + n) * Dm + 128 * k4 + 32 * u + 8 * quad);
        acc[0][nb] = mfma16(av[0][u], bv, acc[0][nb]);
        acc[1][nb] = mfma16(av[1][u], bv, acc[1][nb]);
      }
  }
  // C layout: lane holds gate column 16*nb + n of tokens t0 + 16*a + 4*quad + i
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int j = 16 * nb + n;
    if (j >= J) continue;
    const float b = bf16_to_f32(bias[j]);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = t0 + 16 * a + 4 * quad + i;
        if (t < N) gates[(size_t)t * J + j] = f32_to_bf16(1.0f / (1.0f + __expf(-(acc[a][nb][i] + b))));
      }
  }
}

// dz[tok][j] = dgates * g * (1 - g) for j < J, zero up to column 63 (bf16)
__global__ void g_dz(const bf16_t *__restrict__ gates, const bf16_t *__restrict__ dgates, int N, int J, bf16_t *__restrict__ dz) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)N * JP) return;
  const size_t t = i / JP;
  const int j = (int)(i % JP);
  float v = 0.f;
  if (j < J) {
    const float g = bf16_to_f32(gates[t * J + j]);
    v = bf16_to_f32(dgates[t * J + j]) * g * (1.0f - g);
  }
  dz[i] = f32_to_bf16(v);
}

// dx[tok][dim] += sum_j dz[tok][j] w[dim][j]: MFMA rows = dims (A = padded weights), columns = tokens (B = dz rows).
// 64 dims per step as four matrix instructions whose row r stands for dim 16*(r >> 2) + 4*k + (r & 3) (k = instruction):
// lane (token n, quad) then holds the 16 consecutive dims 16*quad .. +15 of the step, and the four quads of a token
// cover 128 contiguous bytes of its dx row.
__global__ __launch_bounds__(256) void g_dx(const bf16_t *__restrict__ dz, const bf16_t *__restrict__ wp, int N, int Dm,
                                            bf16_t *dx) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int t0 = (blockIdx.x * 4 + wid) * 32;  // two tiles of 16 tokens per wave: every weight operand is used twice
  if (t0 >= N) return;
  int tok[2];
  bf16x8 bz[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    tok[a] = t0 + 16 * a + n;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) bz[a][ks] = tok[a] < N ? ld8(dz + (size_t)tok[a] * JP + 32 * ks + 8 * quad) : zero8();
  }
  const int rdim = 16 * (n >> 2) + (n & 3);  // dim (inside the step) of A row n, before the + 4*k of instruction k
  for (int d0 = 0; d0 < Dm; d0 += 64) {
    f32x4 acc[2][4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bf16_t *wr = wp + (size_t)(d0 + rdim + 4 * k) * JP + 8 * quad;
      const bf16x8 w0 = ld8(wr), w1 = ld8(wr + 32);
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        acc[a][k] = mfma16(w0, bz[a][0], f32x4{0.f, 0.f, 0.f, 0.f});
        acc[a][k] = mfma16(w1, bz[a][1], acc[a][k]);
      }
    }
    // C layout: lane holds rows 4*quad + i of every instruction = dims d0 + 16*quad + 4*k + i of token column n
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      if (tok[a] >= N) continue;
      bf16_t *d = dx + (size_t)tok[a] * Dm + d0 + 16 * quad;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bf16x8 cur = ld8(d + 8 * h);
        bf16x8 r;
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = (__bf16)((float)cur[e] + acc[a][2 * h + (e >> 2)][e & 3]);
        *reinterpret_cast<bf16x8 *>(d + 8 * h) = r;
      }
    }
  }
}

// dW partial: part[chunk][dim][j] = sum over the chunk's tokens of x[tok][dim] dz[tok][j]; a workgroup owns 128 dims
// (wave w the 16-row blocks w and w+4) and all 64 (padded) gate columns.  The next 32-token tile is fetched into
// registers while the current one is consumed.  The workgroups of the first dim tile also produce the chunk's column
// sums of dz (db) with an all-ones A operand.
__global__ __launch_bounds__(256) void g_dw(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dz, int N, int Dm,
                                            int chunk, float *__restrict__ part, float *__restrict__ pb) {
  using GX = TileGeom<128>;
  using GZ = TileGeom<JP>;
  __shared__ __align__(16) bf16_t sx[GX::ROW_ELEMS], sz[GZ::ROW_ELEMS];
  const int d0 = blockIdx.x * 128, s = blockIdx.y;
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const bool sums = blockIdx.x == 0 && wid == 0;
  f32x4 acc[2][JP / 16], csum[JP / 16];
#pragma unroll
  for (int nb = 0; nb < JP / 16; ++nb) {
    acc[0][nb] = acc[1][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    csum[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  bf16x8 ones;
#pragma unroll
  for (int jj = 0; jj < 8; ++jj) ones[jj] = (__bf16)1.0f;
  const int b = s * chunk, e = min(N, b + chunk);
  const int zrow = threadIdx.x / 8, zseg = threadIdx.x % 8;  // dz tile: 32 rows x 8 segments = 256 items
  bf16x8 rx[2], rz;
  auto fetch = [&](int t0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int it = threadIdx.x + 256 * i, t = t0 + it / 16;
      rx[i] = t < e ? ld8(x + (size_t)t * Dm + d0 + 8 * (it % 16)) : zero8();
    }
    rz = t0 + zrow < e ? ld8(dz + (size_t)(t0 + zrow) * JP + 8 * zseg) : zero8();
  };
  if (b < e) fetch(b);
  for (int t0 = b; t0 < e; t0 += 32) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int it = threadIdx.x + 256 * i;
      *reinterpret_cast<bf16x8 *>(sx + GX::row_off(it / 16, it % 16)) = rx[i];
    }
    *reinterpret_cast<bf16x8 *>(sz + GZ::row_off(zrow, zseg)) = rz;
    __syncthreads();
    if (t0 + 32 < e) fetch(t0 + 32);
    bf16x8 av[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) av[a] = lds_tr_operand<128>(sx, wid + 4 * a);
#pragma unroll
    for (int nb = 0; nb < JP / 16; ++nb) {
      const bf16x8 bv = lds_tr_operand<JP>(sz, nb);
#pragma unroll
      for (int a = 0; a < 2; ++a) acc[a][nb] = mfma16(av[a], bv, acc[a][nb]);
      if (sums) csum[nb] = mfma16(ones, bv, csum[nb]);
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
  if (sums && quad == 0) {  // every row of csum holds the column sums; row 0 lives in quad 0
#pragma unroll
    for (int nb = 0; nb < JP / 16; ++nb) pb[(size_t)s * JP + 16 * nb + n] = csum[nb][0];
  }
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

// Forward launches with the transposed weight copy in `wt` (device, ((J+15)/16*16) * d_model bf16).
static int gate_forward_launch(int N, int d_model, int J, const void *x, const void *w, const void *bias, void *gates,
                               bf16_t *wt, hipStream_t s) {
  const int NB = (J + 15) / 16, JR = 16 * NB;
  ProfScope ps(PROF_GATE_FWD, s);
  g_prep_w<<<(unsigned)(((size_t)JR * d_model + 255) / 256), 256, 0, s>>>((const bf16_t *)w, d_model, J, JR, wt, nullptr);
  const unsigned grid = (unsigned)((N + 127) / 128);
  switch (NB) {
    case 1: g_fwd<1><<<grid, 256, 0, s>>>((const bf16_t *)x, wt, (const bf16_t *)bias, N, d_model, J, (bf16_t *)gates); break;
    case 2: g_fwd<2><<<grid, 256, 0, s>>>((const bf16_t *)x, wt, (const bf16_t *)bias, N, d_model, J, (bf16_t *)gates); break;
    case 3: g_fwd<3><<<grid, 256, 0, s>>>((const bf16_t *)x, wt, (const bf16_t *)bias, N, d_model, J, (bf16_t *)gates); break;
    default: g_fwd<4><<<grid, 256, 0, s>>>((const bf16_t *)x, wt, (const bf16_t *)bias, N, d_model, J, (bf16_t *)gates); break;
  }
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

extern "C" int ssa_gate_forward(const ssa_params_t *p, int32_t d_model, const void *x, const void *w, const void *bias,
                                void *gates, void *ws_, size_t ws_bytes, void *stream) {
  int J;
  const int rc = gate_check(p, d_model, &J);
  if (rc != SSA_OK) return rc;
  const int N = p->n_tokens;
  if (N == 0) return SSA_OK;
  if (!x || !w || !bias || !gates) return SSA_ERR_NULL;
  if (!aligned16(x, w, bias, gates)) return SSA_ERR_ALIGNMENT;
  if (!ws_ || ws_bytes < ssa_gate_workspace_bytes(p, d_model, 0)) return SSA_ERR_WORKSPACE;
  const GatePlan pl = gate_plan(N, d_model, J, false);
  char *ws = (char *)align_up((size_t)ws_, 256);
  return gate_forward_launch(N, d_model, J, x, w, bias, gates, (bf16_t *)(ws + pl.wt), (hipStream_t)stream);
}

// ---- the same forward for callers that cannot allocate: the transposed weight copy lives in a static device array.
// Every device the library runs on holds its own copy of the array at its own address; the address is looked up once
// per device (with that device current) and only that pointer is ever handed to a kernel.
constexpr int GATE_STATIC_MAX_DMODEL = 4096;
constexpr size_t GATE_STATIC_BYTES = (size_t)JP * GATE_STATIC_MAX_DMODEL * sizeof(bf16_t);  // 512 KiB
static __device__ __align__(256) unsigned char scratch[GATE_STATIC_BYTES];

constexpr int GATE_MAX_DEVICES = 64;
static std::mutex scratch_mutex;
static void *scratch_ptr[GATE_MAX_DEVICES];  // device address of `scratch` per HIP device, NULL until looked up

static int gate_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= GATE_MAX_DEVICES) return SSA_ERR_HIP;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SSA_ERR_HIP;
    scratch_ptr[dev] = ptr;
  }
  *out = scratch_ptr[dev];
  return SSA_OK;
}

extern "C" int ssa_gate_forward_static(const ssa_params_t *p, int32_t d_model, const void *x, const void *w,
                                       const void *bias, void *gates, void *stream) {
  int J;
  const int rc = gate_check(p, d_model, &J);
  if (rc != SSA_OK) return rc;
  if (d_model > GATE_STATIC_MAX_DMODEL) return SSA_ERR_UNSUPPORTED;  // the static array holds 64 x 4096 weights
  const int N = p->n_tokens;
  if (N == 0) return SSA_OK;
  if (!x || !w || !bias || !gates) return SSA_ERR_NULL;
  if (!aligned16(x, w, bias, gates)) return SSA_ERR_ALIGNMENT;
  void *wt = nullptr;
  const int rs = gate_scratch(&wt);
  if (rs != SSA_OK) return rs;
  return gate_forward_launch(N, d_model, J, x, w, bias, gates, (bf16_t *)wt, (hipStream_t)stream);
}

extern "C" int ssa_gate_backward(const ssa_params_t *p, int32_t d_model, const void *x, const void *w, const void *gates,
                                 const void *dgates, void *dx_accum, float *dw, float *dbias, void *ws_, size_t ws_bytes,
                                 void *stream) {
  int J;
  const int rc = gate_check(p, d_model, &J);
  if (rc != SSA_OK) return rc;
  const int N = p->n_tokens;
  hipStream_t s = (hipStream_t)stream;
  if (N == 0) {  // no tokens: the parameter gradients are zero (a sum over zero partials)
    if (!dw || !dbias) return SSA_ERR_NULL;
    g_sum_parts<<<1, 64, 0, s>>>(nullptr, 0, 1, J, dbias);
    g_sum_parts<<<(unsigned)(((size_t)d_model * J + 255) / 256), 256, 0, s>>>(nullptr, 0, d_model, J, dw);
    return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
  }
  if (!x || !w || !gates || !dgates || !dx_accum || !dw || !dbias) return SSA_ERR_NULL;
  if (!aligned16(x, w, gates, dgates, dx_accum, dw, dbias)) return SSA_ERR_ALIGNMENT;
  if (!ws_ || ws_bytes < ssa_gate_workspace_bytes(p, d_model, 1)) return SSA_ERR_WORKSPACE;
  const GatePlan pl = gate_plan(N, d_model, J, true);
  char *ws = (char *)align_up((size_t)ws_, 256);
  bf16_t *wp = (bf16_t *)(ws + pl.wp), *dz = (bf16_t *)(ws + pl.dz);
  float *pw = (float *)(ws + pl.pw), *pb = (float *)(ws + pl.pb);
  ProfScope ps(PROF_GATE_BWD, s);
  g_prep_w<<<(unsigned)(((size_t)d_model * JP + 255) / 256), 256, 0, s>>>((const bf16_t *)w, d_model, J, 0, nullptr, wp);
  g_dz<<<(unsigned)(((size_t)N * JP + 255) / 256), 256, 0, s>>>((const bf16_t *)gates, (const bf16_t *)dgates, N, J, dz);
  g_dx<<<(unsigned)((N + 127) / 128), 256, 0, s>>>(dz, wp, N, d_model, (bf16_t *)dx_accum);
  g_dw<<<dim3(d_model / 128, pl.chunks), 256, 0, s>>>((const bf16_t *)x, dz, N, d_model, pl.chunk, pw, pb);
  g_sum_parts<<<1, 64, 0, s>>>(pb, pl.chunks, 1, J, dbias);
  g_sum_parts<<<(unsigned)(((size_t)d_model * J + 255) / 256), 256, 0, s>>>(pw, pl.chunks, d_model, J, dw);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}
