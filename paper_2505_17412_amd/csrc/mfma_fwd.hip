// bf16 MFMA forward kernels of SSA (paper eq. (4)-(6), Algorithm 1, window paragraph) for gfx950.
//
// One wavefront owns 16 query rows = (16 / h_s) consecutive sorted tokens x the h_s heads of one KV group and
// keeps their running softmax state in registers (Algorithm 1's m, l, o).  Scores are produced TRANSPOSED
// (S^T = K Q^T, keys x queries) so that the probabilities land in the lanes exactly as the B operand of the
// second contraction O^T = V^T P^T needs them; V is read from a copy stored in chunks of 8 tokens, transposed
// inside each chunk, which makes every MFMA operand one 16-byte load.
#include "mfma_common.h"
#include "topk_device.h"
#include "mfma_launch.h"
#include "profile.h"

namespace {

template <int D>
struct FwdState {
  f32x4 o[D / 16];  // o[dt][i]: output dim 16*dt + 4*quad + i of query column n
  float m, l;       // running max (log2 domain) and this lane's share of the running sum
};

// Scores of one 32-key tile for the wave's 16 queries, scaled into the log2 domain.
// v[j]: key kb + 8*quad + j, query n.
template <int D>
__device__ inline void score_tile(const bf16x8 (&qop)[D / 32], const bf16_t *__restrict__ Kg, size_t kstride, int kb,
                                  float sl2, float (&v)[8]) {
  const int quad = threadIdx.x >> 4 & 3;
  const bf16_t *r0 = Kg + (size_t)tile_key_row(kb, 0) * kstride + 8 * quad;
  const bf16_t *r1 = r0 + 4 * kstride;
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    s0 = mfma16(ld8(r0 + 32 * ks), qop[ks], s0);
    s1 = mfma16(ld8(r1 + 32 * ks), qop[ks], s1);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[i] = s0[i] * sl2;
    v[4 + i] = s1[i] * sl2;
  }
}

// One online-softmax step (Algorithm 1, inner loop body) over a 32-key tile.
template <int D, bool MASK>
__device__ inline void fwd_tile(FwdState<D> &st, const bf16x8 (&qop)[D / 32], const bf16_t *__restrict__ Kg,
                                size_t kstride, const bf16_t *__restrict__ Vtg, size_t vchunk, int kb, int lo, int hi,
                                float sl2) {
  const int n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
  float v[8];
  score_tile<D>(qop, Kg, kstride, kb, sl2, v);
  if (MASK) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int key = kb + 8 * quad + j;
      if (key < lo || key >= hi) v[j] = -INFINITY;
    }
  }
  float tmax = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
  const float mn = fmaxf(st.m, tmax);
  const float ms = mn == -INFINITY ? 0.f : mn;  // nothing seen yet: keep exp2 arguments finite or -inf
  const float alpha = fast_exp2(st.m - ms);
  float psum = 0.f;
  bf16x8 pb;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float p = fast_exp2(v[j] - ms);
    psum += p;
    pb[j] = (__bf16)p;
  }
  st.l = st.l * alpha + psum;
  st.m = mn;
  const bf16_t *vt = Vtg + (size_t)((kb >> 3) + quad) * vchunk + (size_t)n * 8;
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) {
    st.o[dt] *= alpha;
    st.o[dt] = mfma16(ld8(vt + dt * 128), pb, st.o[dt]);
  }
}

// All tiles of the key range [wlo, whi) (wave-uniform); each lane only sees keys inside its own [lo, hi).
template <int D>
__device__ inline void fwd_range(FwdState<D> &st, const bf16x8 (&qop)[D / 32], const bf16_t *Kg, size_t kstride,
                                 const bf16_t *Vtg, size_t vchunk, int wlo, int whi, int lo, int hi, bool uniform,
                                 float sl2) {
  for (int kb = wlo & ~7; kb < whi; kb += 32) {
    if (uniform && kb >= wlo && kb + 32 <= whi) fwd_tile<D, false>(st, qop, Kg, kstride, Vtg, vchunk, kb, lo, hi, sl2);
    else fwd_tile<D, true>(st, qop, Kg, kstride, Vtg, vchunk, kb, lo, hi, sl2);
  }
}

struct FwdArgs {
  MfmaView v;
  const bf16_t *Q;
  bf16_t *Ob;    // [3,N,Hq,D]
  float *lse;    // [3,N,Hq]
  int32_t *idx;  // [N,Hkv,T]
};

struct Row {  // what a lane knows about its query column
  int pos, tok, h;
  bool valid;
};

template <int D>
__device__ inline Row load_query(const FwdArgs &a, int pos0, int g, bf16x8 (&qop)[D / 32]) {
  const int n = threadIdx.x & 15, quad = threadIdx.x >> 4 & 3;
  Row r;
  r.pos = pos0 + n / a.v.hs;
  r.valid = r.pos < a.v.N;
  r.tok = r.valid ? a.v.perm[r.pos] : 0;
  r.h = g * a.v.hs + n % a.v.hs;
  const bf16_t *q = a.Q + ((size_t)r.tok * a.v.Hq + r.h) * D + 8 * quad;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) qop[ks] = r.valid ? ld8(q + 32 * ks) : zero8();
  return r;
}

template <int D>
__device__ inline void init_state(FwdState<D> &st) {
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) st.o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY;
  st.l = 0.f;
}

// Normalise (Algorithm 1: o * exp(m - l)), store the branch output and its log-sum-exp; returns lse in log2 units.
template <int D>
__device__ inline float finish(const FwdArgs &a, FwdState<D> &st, int branch, const Row &r) {
  const int quad = threadIdx.x >> 4 & 3;
  float l = st.l;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  const float inv = l > 0.f ? 1.0f / l : 0.f;
  const float lse2 = l > 0.f ? st.m + __log2f(l) : -INFINITY;
  if (r.valid) {
    bf16_t *o = a.Ob + (((size_t)branch * a.v.N + r.tok) * a.v.Hq + r.h) * D + 4 * quad;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      bf16x4 w;
#pragma unroll
      for (int i = 0; i < 4; ++i) w[i] = (__bf16)(st.o[dt][i] * inv);
      *reinterpret_cast<bf16x4 *>(o + 16 * dt) = w;
    }
    if (quad == 0) a.lse[((size_t)branch * a.v.N + r.tok) * a.v.Hq + r.h] = lse2 * LN2;
  }
  return lse2;
}

// ---- top-k over unsigned fixed-point scores held in LDS by one wavefront (ties -> lowest id) ----
__device__ inline void topk_wave_u32(const uint32_t *S, int n, int T, int base, int32_t *out, uint32_t *sel) {
  const int lane = threadIdx.x & 63;
  const int words = (n + 31) >> 5;
  for (int i = lane; i < words; i += 64) sel[i] = 0u;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int rounds = T < n ? T : n;
  for (int r = 0; r < rounds; ++r) {
    uint64_t best = 0ull;
    for (int j = lane; j < n; j += 64) {
      if ((sel[j >> 5] >> (j & 31)) & 1u) continue;
      const uint64_t key = ((uint64_t)S[j] << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)j);
      best = key > best ? key : best;
    }
    best = wave_max_u64(best);
    const uint32_t j = 0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull);
    if (lane == 0) sel[j >> 5] |= 1u << (j & 31);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  int written = 0;
  for (int j0 = 0; j0 < n; j0 += 64) {
    const int j = j0 + lane;
    const bool s = j < n && ((sel[j >> 5] >> (j & 31)) & 1u);
    const uint64_t m = __ballot(s);
    if (s) out[written + __popcll(m & ((1ull << lane) - 1ull))] = base + j;
    written += __popcll(m);
  }
  for (int w = written + lane; w < T; w += 64) out[w] = -1;
}

constexpr float SCORE_FIX = 134217728.0f;  // 2^27: a row's scores sum to h_s <= 16 < 2^5

// Compression branch (eq. (4) first term over the mean-pooled keys of eq. (5)), then the selection scores of
// eq. (6) accumulated per selection block in LDS as fixed-point integers (integer adds commute, so the result
// does not depend on scheduling), then the top-k.
template <int D>
__global__ __launch_bounds__(256) void m_cmp_fwd(FwdArgs a) {
  extern __shared__ uint32_t lds[];
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int hs = a.v.hs, tpw = 16 / hs, g = blockIdx.y;
  const int pos0 = (blockIdx.x * 4 + wid) * tpw;
  if (pos0 >= a.v.N) return;
  bf16x8 qop[D / 32];
  const Row r = load_query<D>(a, pos0, g, qop);
  const int item = r.valid ? a.v.tok_item[r.pos] : 0;
  const int lo = r.valid ? a.v.cmp_batch[item] : 0, hi = r.valid ? a.v.cmp_batch[item + 1] : 0;
  const int wlo = wave_min_i(r.valid ? lo : 0x7fffffff), whi = wave_max_i(hi);
  const bool uniform = __all(r.valid && lo == wlo && hi == whi);
  const size_t kstride = (size_t)a.v.Hkv * D, vchunk = kstride * 8;
  const bf16_t *Kg = a.v.Kc + (size_t)g * D, *Vtg = a.v.Vct + (size_t)g * D * 8;
  FwdState<D> st;
  init_state(st);
  fwd_range<D>(st, qop, Kg, kstride, Vtg, vchunk, wlo, whi, lo, hi, uniform, a.v.sl2);
  const float lse2 = finish<D>(a, st, 0, r);
  if (!a.idx) return;

  // ---- selection scores, eq. (6)
  const int s_max = a.v.s_max;
  uint32_t *S = lds + (size_t)wid * tpw * s_max;
  uint32_t *sel = lds + (size_t)4 * tpw * s_max + (size_t)wid * ((s_max + 31) >> 5);
  for (int i = lane; i < tpw * s_max; i += 64) S[i] = 0u;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int s0 = r.valid ? a.v.slc_batch[item] : 0;
  uint32_t *Srow = S + (size_t)(n / hs) * s_max;
  for (int kb = wlo & ~7; kb < whi; kb += 32) {
    float v[8];
    score_tile<D>(qop, Kg, kstride, kb, a.v.sl2, v);
    float p[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int key = kb + 8 * quad + j;
      p[j] = (key >= lo && key < hi) ? fast_exp2(v[j] - lse2) : 0.f;
      for (int off = 1; off < hs; off <<= 1) p[j] += __shfl_xor(p[j], off);  // sum over the group's heads
    }
    if (r.valid && (n % hs) == 0) {
      int cur = -1;
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int key = kb + 8 * quad + j;
        if (key >= lo && key < hi) {
          const int b = a.v.cmp_slc[key] - s0;
          if (b != cur) {
            if (cur >= 0) atomicAdd(&Srow[cur], (uint32_t)(acc * SCORE_FIX));
            cur = b;
            acc = 0.f;
          }
          acc += p[j];
        }
      }
      if (cur >= 0) atomicAdd(&Srow[cur], (uint32_t)(acc * SCORE_FIX));
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  // ---- top-k, one token of the wave after the other
  for (int tl = 0; tl < tpw; ++tl) {
    const int pos = pos0 + tl;
    if (pos >= a.v.N) break;
    const int tok = a.v.perm[pos], it = a.v.tok_item[pos];
    const int b0 = a.v.slc_batch[it], nb = a.v.slc_batch[it + 1] - b0;
    topk_wave_u32(S + (size_t)tl * s_max, nb, a.v.T, b0, a.idx + ((size_t)tok * a.v.Hkv + g) * a.v.T, sel);
  }
}

// Selection branch: Algorithm 1.  The wave's tokens walk the union of their selected blocks in ascending id;
// a token that did not select the current block sees it fully masked.
template <int D>
__global__ __launch_bounds__(256) void m_slc_fwd(FwdArgs a) {
  const int wid = threadIdx.x >> 6;
  const int hs = a.v.hs, tpw = 16 / hs, g = blockIdx.y, T = a.v.T;
  const int pos0 = (blockIdx.x * 4 + wid) * tpw;
  if (pos0 >= a.v.N) return;
  bf16x8 qop[D / 32];
  const Row r = load_query<D>(a, pos0, g, qop);
  const size_t kstride = (size_t)a.v.Hkv * D, vchunk = kstride * 8;
  const bf16_t *Kg = a.v.Ks + (size_t)g * D, *Vtg = a.v.Vt + (size_t)g * D * 8;
  const int32_t *row = a.idx + ((size_t)r.tok * a.v.Hkv + g) * T;
  FwdState<D> st;
  init_state(st);
  int j = 0;
  for (;;) {
    const int cur = (r.valid && j < T) ? row[j] : -1;
    const int key = cur < 0 ? 0x7fffffff : cur;
    const int b = wave_min_i(key);
    if (b == 0x7fffffff) break;
    const bool sel = key == b;
    if (sel) ++j;
    const int bs = a.v.slc_start[b], be = a.v.slc_start[b + 1];
    fwd_range<D>(st, qop, Kg, kstride, Vtg, vchunk, bs, be, sel ? bs : 0, sel ? be : 0, __all(sel), a.v.sl2);
  }
  finish<D>(a, st, 1, r);
}

// Window branch: keys are the tokens of the query's own window.
template <int D>
__global__ __launch_bounds__(256) void m_win_fwd(FwdArgs a) {
  const int wid = threadIdx.x >> 6;
  const int hs = a.v.hs, tpw = 16 / hs, g = blockIdx.y;
  const int pos0 = (blockIdx.x * 4 + wid) * tpw;
  if (pos0 >= a.v.N) return;
  bf16x8 qop[D / 32];
  const Row r = load_query<D>(a, pos0, g, qop);
  const int w = r.valid ? a.v.tok_win[r.pos] : 0;
  const int lo = r.valid ? a.v.win_start[w] : 0, hi = r.valid ? a.v.win_start[w + 1] : 0;
  const int wlo = wave_min_i(r.valid ? lo : 0x7fffffff), whi = wave_max_i(hi);
  const bool uniform = __all(r.valid && lo == wlo && hi == whi);
  const size_t kstride = (size_t)a.v.Hkv * D, vchunk = kstride * 8;
  FwdState<D> st;
  init_state(st);
  fwd_range<D>(st, qop, a.v.Ks + (size_t)g * D, kstride, a.v.Vt + (size_t)g * D * 8, vchunk, wlo, whi, lo, hi, uniform,
               a.v.sl2);
  finish<D>(a, st, 2, r);
}

// eq. (4): out = sum_b gate_b * out_b, 8 elements per thread.
__global__ void m_combine(const bf16_t *__restrict__ Ob, const bf16_t *__restrict__ gates, size_t rows /*N*Hq*/, int D,
                          bf16_t *__restrict__ out) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one 8-element chunk
  const int per_row = D / 8;
  if (i >= rows * per_row) return;
  const size_t row = i / per_row;
  const size_t off = row * D + (i % per_row) * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int b = 0; b < 3; ++b) {
    const float w = bf16_to_f32(gates[row * 3 + b]);
    const bf16x8 x = ld8(Ob + (size_t)b * rows * D + off);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += w * (float)x[j];
  }
  bf16x8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (__bf16)acc[j];
  *reinterpret_cast<bf16x8 *>(out + off) = o;
}

template <int D>
int launch_forward(const FwdArgs &a, const bf16_t *gates, bf16_t *out, size_t lds_bytes, hipStream_t s) {
  const int tpw = 16 / a.v.hs;
  const dim3 grid((a.v.N + 4 * tpw - 1) / (4 * tpw), a.v.Hkv);
  {
    ProfScope ps(PROF_CMP_FWD, s);
    m_cmp_fwd<D><<<grid, 256, lds_bytes, s>>>(a);
  }
  {
    ProfScope ps(PROF_SLC_FWD, s);
    m_slc_fwd<D><<<grid, 256, 0, s>>>(a);
  }
  {
    ProfScope ps(PROF_WIN_FWD, s);
    m_win_fwd<D><<<grid, 256, 0, s>>>(a);
  }
  {
    ProfScope ps(PROF_COMBINE, s);
    const size_t chunks = (size_t)a.v.N * a.v.Hq * (D / 8);
    m_combine<<<(unsigned)((chunks + 255) / 256), 256, 0, s>>>(a.Ob, gates, (size_t)a.v.N * a.v.Hq, D, out);
  }
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

}  // namespace

size_t mfma_cmp_lds_bytes(int hs, int s_max) {
  const int tpw = 16 / hs;
  return ((size_t)4 * tpw * s_max + (size_t)4 * ((s_max + 31) / 32) + 16) * sizeof(uint32_t);
}

int mfma_forward_kernels(const MfmaView &v, int D, const void *q, const void *gates, void *out, float *lse,
                         int32_t *idx, void *out_branch, hipStream_t s) {
  FwdArgs a{v, (const bf16_t *)q, (bf16_t *)out_branch, lse, idx};
  const size_t lds = mfma_cmp_lds_bytes(v.hs, v.s_max);
  switch (D) {
    case 32: return launch_forward<32>(a, (const bf16_t *)gates, (bf16_t *)out, lds, s);
    case 64: return launch_forward<64>(a, (const bf16_t *)gates, (bf16_t *)out, lds, s);
    case 128: return launch_forward<128>(a, (const bf16_t *)gates, (bf16_t *)out, lds, s);
    default: return SSA_ERR_UNSUPPORTED;
  }
}
