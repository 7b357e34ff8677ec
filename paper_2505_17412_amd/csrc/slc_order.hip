// Token order of the selection-branch kernels (gfx950).
//
// The query-centric selection kernels (Algorithm 1 forward, and the selection part of dQ) give a wavefront 16/h_s
// tokens and a workgroup 4 wavefronts, and walk the UNION of the blocks those tokens selected: every block in the union
// costs the wavefront a full tile pass, whichever of its tokens selected it.  Which tokens share a wavefront is free to
// choose (each token's result is exact whatever its neighbours are), so tokens with similar selections are put next to
// each other: per KV head, tokens are ordered by the bit mask "which of the ~16 most often selected blocks did I
// select" (stable, so the spatial order survives inside equal masks).  On the benchmark workload 16 blocks take almost
// half of all selections, and this order shrinks the union of a token pair from 26.9 to 23.1 blocks and that of a
// workgroup from 56 to 47.  Integer work only; the order, and with it every result, is deterministic.
#include "mfma_launch.h"
#include "profile.h"

namespace {

constexpr int POP_MAX = 16;              // at most this many blocks get a mask bit
constexpr uint32_t TAKEN = 0xFFFFFFFFu;  // count of a block that already has a rank

__global__ void o_fill(uint32_t *p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// counts[g][b] = how many (token, g) rows selected block b.  A workgroup histograms its share of the index tensor in
// LDS (bins <= LDS_BINS) and adds the non-zero bins to memory; integer adds commute, so the result is exact.
constexpr int LDS_BINS = 8192;
__global__ __launch_bounds__(256) void o_count(const int32_t *__restrict__ idx, size_t entries, int Hkv, int T, int Ns,
                                               uint32_t *__restrict__ counts) {
  extern __shared__ uint32_t hist[];
  const int bins = Hkv * Ns;
  const bool local = bins <= LDS_BINS;
  if (local) {
    for (int i = threadIdx.x; i < bins; i += 256) hist[i] = 0u;
    __syncthreads();
  }
  const size_t per = (entries + gridDim.x - 1) / gridDim.x;
  const size_t begin = (size_t)blockIdx.x * per, end = begin + per < entries ? begin + per : entries;
  for (size_t e = begin + threadIdx.x; e < end; e += 256) {
    const int b = idx[e];
    if (b < 0 || b >= Ns) continue;
    const int g = (int)(e / T % Hkv);
    if (local) atomicAdd(&hist[g * Ns + b], 1u); else atomicAdd(&counts[(size_t)g * Ns + b], 1u);
  }
  if (local) {
    __syncthreads();
    for (int i = threadIdx.x; i < bins; i += 256)
      if (hist[i]) atomicAdd(&counts[i], hist[i]);
  }
}

// rank[g][b] = 0 .. pop-1 for the pop most selected blocks of KV head g (ties to the lower id), -1 otherwise.
// One workgroup per KV head; counts are consumed (ranked blocks are marked TAKEN).
__global__ __launch_bounds__(256) void o_rank(uint32_t *__restrict__ counts, int Ns, int pop, int32_t *__restrict__ rank) {
  __shared__ unsigned long long best[4];
  uint32_t *cnt = counts + (size_t)blockIdx.x * Ns;
  int32_t *rk = rank + (size_t)blockIdx.x * Ns;
  for (int r = 0; r < pop; ++r) {
    unsigned long long b = 0ull;
    for (int j = threadIdx.x; j < Ns; j += 256) {
      const uint32_t c = cnt[j];
      if (c == TAKEN || c == 0u) continue;
      const unsigned long long key = ((unsigned long long)c << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)j);
      b = key > b ? key : b;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const unsigned long long o = __shfl_xor(b, off);
      b = o > b ? o : b;
    }
    if ((threadIdx.x & 63) == 0) best[threadIdx.x >> 6] = b;
    __syncthreads();
    unsigned long long w = best[0];
    for (int i = 1; i < 4; ++i) w = best[i] > w ? best[i] : w;
    __syncthreads();  // best[] is rewritten in the next round
    if (w == 0ull) break;  // fewer than pop blocks were selected at all (uniform: every thread sees the same w)
    const uint32_t j = 0xFFFFFFFFu - (uint32_t)(w & 0xFFFFFFFFull);
    if (threadIdx.x == 0) { rk[j] = r; cnt[j] = TAKEN; }
    __syncthreads();
  }
}

// Item i = g*N + pos (sorted position): key = (g << pop) | mask, value = the token's caller index.
__global__ void o_keys(const int32_t *__restrict__ idx, const int32_t *__restrict__ perm, const int32_t *__restrict__ rank,
                       int N, int Hkv, int T, int Ns, int pop, uint64_t *__restrict__ keys, uint32_t *__restrict__ vals) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)N * Hkv) return;
  const int g = (int)(i / N), pos = (int)(i % N), tok = perm[pos];
  const int32_t *row = idx + ((size_t)tok * Hkv + g) * T;
  uint32_t mask = 0u;
  for (int j = 0; j < T; ++j) {
    const int b = row[j];
    if (b < 0 || b >= Ns) continue;
    const int r = rank[(size_t)g * Ns + b];
    if (r >= 0) mask |= 1u << (pop - 1 - r);
  }
  keys[i] = ((uint64_t)g << pop) | mask;
  vals[i] = (uint32_t)tok;
}

struct OrderPlan {
  size_t counts, rank, k0, k1, v0, v1, aux, total;
};
OrderPlan order_plan(int N, int Hkv, int Ns) {
  OrderPlan p{};
  const size_t items = (size_t)N * Hkv;
  size_t off = 0;
  auto take = [&](size_t n) { const size_t r = off; off += align_up(n, 256); return r; };
  p.counts = take((size_t)Hkv * Ns * 4);
  p.rank = take((size_t)Hkv * Ns * 4);
  p.k0 = take(items * 8); p.k1 = take(items * 8);
  p.v0 = take(items * 4); p.v1 = take(items * 4);
  p.aux = take(sort_pairs_aux_bytes((int)items));
  p.total = off;
  return p;
}

}  // namespace

bool slc_order_wanted(int N, int Hkv) { return N >= SLC_ORDER_MIN_TOKENS && (long long)N * Hkv < (1ll << 30); }

size_t slc_order_workspace(int N, int Hkv, int Ns) { return slc_order_wanted(N, Hkv) ? order_plan(N, Hkv, Ns).total : 0; }

int slc_order_build(const int32_t *idx, const int32_t *perm, int N, int Hkv, int T, int Ns, void *ws_, hipStream_t s,
                    const int32_t **order) {
  *order = nullptr;
  if (!slc_order_wanted(N, Hkv)) return SSA_OK;
  ProfScope ps(PROF_SLC_ORDER, s);
  const OrderPlan p = order_plan(N, Hkv, Ns);
  char *ws = (char *)ws_;
  uint32_t *counts = (uint32_t *)(ws + p.counts);
  int32_t *rank = (int32_t *)(ws + p.rank);
  uint64_t *k0 = (uint64_t *)(ws + p.k0), *k1 = (uint64_t *)(ws + p.k1);
  uint32_t *v0 = (uint32_t *)(ws + p.v0), *v1 = (uint32_t *)(ws + p.v1);
  const size_t bins = (size_t)Hkv * Ns, entries = (size_t)N * Hkv * T, items = (size_t)N * Hkv;
  o_fill<<<64, 256, 0, s>>>(counts, bins, 0u);
  o_fill<<<64, 256, 0, s>>>((uint32_t *)rank, bins, 0xFFFFFFFFu);  // -1
  const size_t lds = bins <= (size_t)LDS_BINS ? bins * 4 : 0;
  o_count<<<512, 256, lds, s>>>(idx, entries, Hkv, T, Ns, counts);
  // mask bits + KV-head bits fill whole 8-bit sort passes: 16 bits (two passes) up to 256 KV heads
  int gbits = 0;
  while ((1 << gbits) < Hkv) ++gbits;
  const int pop = gbits <= 8 ? POP_MAX - gbits : 8;
  o_rank<<<Hkv, 256, 0, s>>>(counts, Ns, pop, rank);
  o_keys<<<(unsigned)((items + 255) / 256), 256, 0, s>>>(idx, perm, rank, N, Hkv, T, Ns, pop, k0, v0);
  const int where = sort_pairs(k0, v0, k1, v1, ws + p.aux, (int)items, pop + gbits, s);
  if (hipGetLastError() != hipSuccess) return SSA_ERR_HIP;
  *order = (const int32_t *)(where ? v1 : v0);
  return SSA_OK;
}
