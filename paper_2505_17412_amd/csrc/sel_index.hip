// Inverse of the selection (gfx950): for every (KV head, selection block) the ascending list of sorted positions of the
// query tokens whose row of the index tensor I (Algorithm 1) holds the block, and the cuts of every list into work chunks.  Built from a bit matrix (integer OR: order independent), then
// compacted in order: integer work only, deterministic.  The block-centric selection kernels (forward and dQ) and the
// key-centric dK/dV kernel walk these lists.
#include "mfma_launch.h"

namespace {

__global__ void m_fill_u32(uint32_t *p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void m_sel_bits(const int32_t *__restrict__ idx, const int32_t *__restrict__ perm, int N, int Hkv, int T, int Ns,
                           int words, uint32_t *bits) {
  const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (size_t)N * Hkv * T) return;
  const int pos = (int)(e / ((size_t)Hkv * T)), g = (int)(e / T % Hkv), j = (int)(e % T);
  const int b = idx[((size_t)perm[pos] * Hkv + g) * T + j];
  if (b < 0 || b >= Ns) return;
  atomicOr(&bits[((size_t)g * Ns + b) * words + (pos >> 5)], 1u << (pos & 31));
}

// The same bit matrix built tile by tile in LDS: workgroup (chunk, g) owns `cw` words = 32*cw sorted positions of all
// Ns blocks of KV head g, sets the bits with LDS atomics and writes every word of its tile (so the matrix needs no
// clearing beforehand).  Needs Ns * cw * 4 bytes of LDS.
__global__ __launch_bounds__(256) void m_sel_bits_tile(const int32_t *__restrict__ idx, const int32_t *__restrict__ perm, int N,
                                                       int Hkv, int T, int Ns, int words, int cw, uint32_t *__restrict__ bits) {
  extern __shared__ __align__(16) unsigned char sel_smem[];
  uint32_t *tile = (uint32_t *)sel_smem;  // [Ns][cw]
  const int g = blockIdx.y, w0 = blockIdx.x * cw, p0 = w0 * 32;
  for (int i = threadIdx.x; i < Ns * cw; i += 256) tile[i] = 0u;
  __syncthreads();
  const int npos = min(32 * cw, N - p0);
  for (int e = threadIdx.x; e < npos * T; e += 256) {
    const int pl = e / T, j = e % T;
    const int b = idx[((size_t)perm[p0 + pl] * Hkv + g) * T + j];
    if (b >= 0 && b < Ns) atomicOr(&tile[b * cw + (pl >> 5)], 1u << (pl & 31));
  }
  __syncthreads();
  const int wn = min(cw, words - w0);
  for (int i = threadIdx.x; i < Ns * cw; i += 256) {
    const int b = i / cw, w = i % cw;
    if (w < wn) bits[((size_t)g * Ns + b) * words + w0 + w] = tile[i];
  }
}

__global__ __launch_bounds__(256) void m_sel_count(const uint32_t *__restrict__ bits, int words, uint32_t *counts) {
  __shared__ uint32_t part[4];
  const uint32_t *row = bits + (size_t)blockIdx.x * words;
  uint32_t c = 0;
  for (int i = threadIdx.x; i < words; i += 256) c += __popc(row[i]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) counts[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// single workgroup: from the per-(g, block) selector counts, four exclusive prefix sums over the n keys:
// start (list offsets), chunk_start (work chunks of chunk_len query tokens), part_row_start (rows of partial sums:
// chunks x keys of the block), bc_chunk_start (work chunks of bc_chunk_len query tokens).
__global__ void m_scan_counts(const uint32_t *counts, int n, int Ns, int chunk_len, int bc_chunk_len, const int32_t *slc_start,
                              int32_t *start, int32_t *chunk_start, int32_t *part_row_start, int32_t *bc_chunk_start) {
  __shared__ uint32_t part[4][1024];
  const int tid = threadIdx.x;
  const int per = (n + 1023) / 1024;
  const int b = min(n, tid * per), e = min(n, b + per);
  uint32_t s[4] = {0u, 0u, 0u, 0u};
  for (int i = b; i < e; ++i) {
    const uint32_t c = counts[i], nch = (c + chunk_len - 1) / chunk_len;
    const int blk = i % Ns;
    s[0] += c; s[1] += nch; s[2] += nch * (uint32_t)(slc_start[blk + 1] - slc_start[blk]);
    s[3] += (c + bc_chunk_len - 1) / bc_chunk_len;
  }
  for (int x = 0; x < 4; ++x) part[x][tid] = s[x];
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    uint32_t v[4];
    for (int x = 0; x < 4; ++x) v[x] = tid >= off ? part[x][tid - off] : 0u;
    __syncthreads();
    for (int x = 0; x < 4; ++x) part[x][tid] += v[x];
    __syncthreads();
  }
  uint32_t run[4];
  for (int x = 0; x < 4; ++x) run[x] = part[x][tid] - s[x];
  for (int i = b; i < e; ++i) {
    const uint32_t c = counts[i], nch = (c + chunk_len - 1) / chunk_len;
    const int blk = i % Ns;
    start[i] = (int32_t)run[0]; chunk_start[i] = (int32_t)run[1]; part_row_start[i] = (int32_t)run[2];
    bc_chunk_start[i] = (int32_t)run[3];
    run[0] += c; run[1] += nch; run[2] += nch * (uint32_t)(slc_start[blk + 1] - slc_start[blk]);
    run[3] += (c + bc_chunk_len - 1) / bc_chunk_len;
  }
  if (tid == 1023) {
    start[n] = (int32_t)part[0][1023]; chunk_start[n] = (int32_t)part[1][1023]; part_row_start[n] = (int32_t)part[2][1023];
    bc_chunk_start[n] = (int32_t)part[3][1023];
  }
}

__global__ __launch_bounds__(256) void m_sel_fill(const uint32_t *__restrict__ bits, int words,
                                                  const int32_t *__restrict__ start, int32_t *list) {
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t base;
  const uint32_t *row = bits + (size_t)blockIdx.x * words;
  if (threadIdx.x == 0) base = (uint32_t)start[blockIdx.x];
  __syncthreads();
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  for (int i0 = 0; i0 < words; i0 += 256) {
    const int i = i0 + threadIdx.x;
    uint32_t w = i < words ? row[i] : 0u;
    const uint32_t c = __popc(w);
    uint32_t incl = c;  // inclusive scan inside the wavefront
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
    if (lane == 63) wsum[wid] = incl;
    __syncthreads();
    uint32_t off = base + incl - c;
    for (int ww = 0; ww < wid; ++ww) off += wsum[ww];
    while (w) {
      const int bit = __ffs(w) - 1;
      list[off++] = i * 32 + bit;
      w &= w - 1;
    }
    __syncthreads();
    if (threadIdx.x == 0) base += wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
  }
}

// Execution order of the work chunks of one chunking: chunks sorted by (KV head, first query position of the chunk), in
// buckets of `bucket` positions (counting sort in LDS, one workgroup).  Chunks that run at the same time then belong to
// different blocks but to the same stretch of tokens, whose query rows they all gather: the rows are fetched into the
// L2 once instead of once per selected block.  The order only decides WHEN a chunk runs, never what it computes, so the
// arbitrary order inside a bucket (LDS atomics) does not touch any result.  order[i] = chunk id; total = chunk_start[n].
constexpr int ORDER_BINS = 8192, ORDER_CS = 4096;
__global__ __launch_bounds__(1024) void m_chunk_order(const int32_t *__restrict__ start, const int32_t *__restrict__ chunk_start,
                                                      const int32_t *__restrict__ list, int n, int Ns, int chunk_len,
                                                      int bucket, int bins_per_head, int32_t *__restrict__ order) {
  __shared__ uint32_t bin[ORDER_BINS];
  __shared__ int32_t cs_lds[ORDER_CS];  // copy of the chunk prefix sums when they fit: the bisections then stay in LDS
  const int nbins = (n / Ns) * bins_per_head;
  const bool in_lds = n + 1 <= ORDER_CS;
  for (int i = threadIdx.x; i < nbins; i += 1024) bin[i] = 0u;
  if (in_lds)
    for (int i = threadIdx.x; i <= n; i += 1024) cs_lds[i] = chunk_start[i];
  __syncthreads();
  const int total = chunk_start[n];
  // chunk w -> its key by bisection over the chunk prefix sums, then the bucket of the chunk's first query position
  auto bin_of = [&](int w) {
    int lo = 0, hi = n;  // chunk_start[lo] <= w < chunk_start[hi]
    if (in_lds) {
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cs_lds[mid] <= w) lo = mid; else hi = mid;
      }
      return (lo / Ns) * bins_per_head + list[start[lo] + (w - cs_lds[lo]) * chunk_len] / bucket;
    }
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (chunk_start[mid] <= w) lo = mid; else hi = mid;
    }
    return (lo / Ns) * bins_per_head + list[start[lo] + (w - chunk_start[lo]) * chunk_len] / bucket;
  };
  for (int w = threadIdx.x; w < total; w += 1024) atomicAdd(&bin[bin_of(w)], 1u);
  __syncthreads();
  {  // exclusive scan of the counters: every thread owns 8 consecutive bins
    __shared__ uint32_t part[1024];
    const int b0 = threadIdx.x * (ORDER_BINS / 1024);
    uint32_t own = 0;
    for (int i = 0; i < ORDER_BINS / 1024; ++i) own += b0 + i < nbins ? bin[b0 + i] : 0u;
    part[threadIdx.x] = own;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      const uint32_t v = (int)threadIdx.x >= off ? part[threadIdx.x - off] : 0u;
      __syncthreads();
      part[threadIdx.x] += v;
      __syncthreads();
    }
    uint32_t run = part[threadIdx.x] - own;
    for (int i = 0; i < ORDER_BINS / 1024; ++i)
      if (b0 + i < nbins) { const uint32_t c = bin[b0 + i]; bin[b0 + i] = run; run += c; }
  }
  __syncthreads();
  for (int w = threadIdx.x; w < total; w += 1024) order[atomicAdd(&bin[bin_of(w)], 1u)] = w;
}

struct Plan { size_t bits, counts, start, list, cstart, prow, bcstart, bcorder, order, total; };

Plan plan(int N, int Hkv, int T, int Ns) {
  Plan p{};
  size_t off = 0;
  auto take = [&](size_t n) { size_t r = off; off += align_up(n, 256); return r; };
  const size_t keys = (size_t)Hkv * Ns, words = ((size_t)N + 31) / 32, entries = (size_t)N * Hkv * T;
  p.bits = take(keys * words * 4); p.counts = take(keys * 4 + 4); p.start = take((keys + 1) * 4);
  p.list = take(entries * 4);
  p.cstart = take((keys + 1) * 4); p.prow = take((keys + 1) * 4); p.bcstart = take((keys + 1) * 4);
  // at most one partly filled chunk per key on top of the full ones (chunks of at least 256 tokens)
  p.bcorder = take((entries / 256 + keys + 8) * 4); p.order = take((entries / 256 + keys + 8) * 4);
  p.total = off;
  return p;
}

}  // namespace

size_t sel_index_bytes(int N, int Hkv, int T, int Ns) { return plan(N, Hkv, T, Ns).total; }

SelIndex sel_index_carve(void *ws_, int N, int Hkv, int T, int Ns, int chunk_len, int bc_chunk_len) {
  const Plan p = plan(N, Hkv, T, Ns);
  char *ws = (char *)ws_;
  SelIndex x{};
  x.bits = (uint32_t *)(ws + p.bits); x.counts = (uint32_t *)(ws + p.counts); x.start = (int32_t *)(ws + p.start);
  x.list = (int32_t *)(ws + p.list);
  x.chunk_start = (int32_t *)(ws + p.cstart); x.part_row_start = (int32_t *)(ws + p.prow);
  x.bc_chunk_start = (int32_t *)(ws + p.bcstart);
  x.bc_order = (int32_t *)(ws + p.bcorder); x.order = (int32_t *)(ws + p.order);
  x.chunk_len = chunk_len; x.bc_chunk_len = bc_chunk_len;
  return x;
}

int sel_index_build(const int32_t *idx, const int32_t *perm, const int32_t *slc_start, int N, int Hkv, int T, int Ns,
                    const SelIndex &x, bool want_dkv_order, hipStream_t s) {
  const int words = (N + 31) / 32, keys = Hkv * Ns;
  // bit matrix: tiles of up to 32 words per block row held in LDS (64 KB), or global atomics when a KV head has more
  // than 16 384 blocks
  int cw = Ns > 0 ? 16384 / Ns : 0;
  if (cw > 32) cw = 32;
  if (cw >= 1) {
    m_sel_bits_tile<<<dim3((words + cw - 1) / cw, Hkv), 256, (size_t)Ns * cw * 4, s>>>(idx, perm, N, Hkv, T, Ns, words, cw, x.bits);
  } else {
    m_fill_u32<<<1024, 256, 0, s>>>(x.bits, (size_t)keys * words, 0u);
    const size_t entries = (size_t)N * Hkv * T;
    m_sel_bits<<<(unsigned)((entries + 255) / 256), 256, 0, s>>>(idx, perm, N, Hkv, T, Ns, words, x.bits);
  }
  m_sel_count<<<keys, 256, 0, s>>>(x.bits, words, x.counts);
  m_scan_counts<<<1, 1024, 0, s>>>(x.counts, keys, Ns, x.chunk_len, x.bc_chunk_len, slc_start, x.start, x.chunk_start,
                                   x.part_row_start, x.bc_chunk_start);
  m_sel_fill<<<keys, 256, 0, s>>>(x.bits, words, x.start, x.list);
  // execution orders of both chunkings; bucket width so that Hkv * ceil(N / bucket) bins fit the LDS table
  int bucket = 64;
  while ((long long)Hkv * ((N + bucket - 1) / bucket) > ORDER_BINS) bucket *= 2;
  const int bph = (N + bucket - 1) / bucket;
  m_chunk_order<<<1, 1024, 0, s>>>(x.start, x.bc_chunk_start, x.list, keys, Ns, x.bc_chunk_len, bucket, bph, x.bc_order);
  if (want_dkv_order)
    m_chunk_order<<<1, 1024, 0, s>>>(x.start, x.chunk_start, x.list, keys, Ns, x.chunk_len, bucket, bph, x.order);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}
