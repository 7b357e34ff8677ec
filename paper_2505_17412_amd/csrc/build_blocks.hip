// Block partition, token sort and block start arrays for SSA on gfx950.
//
// Paper, Sec. "Spatial Sparse Attention": tokens whose voxels fall into the same m^3 sub-grid form a block;
// tokens are sorted by block and the first-token index of every block (array C of Algorithm 1) is kept.
// Here one Morton-order sort serves the three block granularities (all sides are powers of two, so every
// aligned cube is a contiguous run of the Morton order): key = (batch item << 3*bits) | Morton(x,y,z).
// Integer work only; results are bit-exact and independent of scheduling (stable LSD radix sort, no
// order-dependent atomics).
#include "ssa_internal.h"

namespace {

constexpr int SORT_TILE = 256;  // one key per thread, 4 wavefronts per workgroup

enum { META_ERR = 0, META_NC, META_NS, META_NW, META_SMAX, META_CMAX, META_SLC_TOK, META_WIN_TOK, META_CMP_TOK, META_N };

// Spread the low 10 bits of v so that bit i lands on bit 3i.
__device__ inline uint32_t spread3(uint32_t v) {
  v &= 0x3FFu;
  v = (v | (v << 16)) & 0x030000FFu;
  v = (v | (v << 8)) & 0x0300F00Fu;
  v = (v | (v << 4)) & 0x030C30C3u;
  v = (v | (v << 2)) & 0x09249249u;
  return v;
}

__global__ void k_make_keys(const int32_t *__restrict__ coords, const int32_t *__restrict__ offs, int N, int B, int G,
                            int bits, uint64_t *__restrict__ keys, uint32_t *__restrict__ vals, int32_t *meta) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  for (int j = i; j <= B; j += gridDim.x * blockDim.x) {
    const int o = offs[j];
    const bool bad = (j == 0 && o != 0) || (j == B && o != N) || (j > 0 && o < offs[j - 1]) || o < 0 || o > N;
    if (bad) atomicOr(&meta[META_ERR], 1);
  }
  if (i >= N) return;
  int lo = 0, hi = B;  // offs[lo] <= i < offs[hi] for valid offsets
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (offs[mid] <= i) lo = mid; else hi = mid;
  }
  int x = coords[3 * i], y = coords[3 * i + 1], z = coords[3 * i + 2];
  if ((unsigned)x >= (unsigned)G || (unsigned)y >= (unsigned)G || (unsigned)z >= (unsigned)G) {
    atomicOr(&meta[META_ERR], 2);
    x = y = z = 0;
  }
  const uint64_t code = (uint64_t)((spread3((uint32_t)x) << 2) | (spread3((uint32_t)y) << 1) | spread3((uint32_t)z));
  keys[i] = ((uint64_t)lo << (3 * bits)) | code;
  vals[i] = (uint32_t)i;
}

// Per-tile digit histogram, stored digit-major so that one linear scan yields the scatter offsets.
__global__ void k_sort_hist(const uint64_t *__restrict__ keys, int N, int shift, int nTiles, uint32_t *__restrict__ hist) {
  __shared__ uint32_t h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int i = blockIdx.x * SORT_TILE + threadIdx.x;
  if (i < N) atomicAdd(&h[(uint32_t)(keys[i] >> shift) & 255u], 1u);
  __syncthreads();
  hist[threadIdx.x * nTiles + blockIdx.x] = h[threadIdx.x];
}

// Exclusive prefix sum over the `n` threads of a workgroup (n <= 1024 a multiple of 64): returns the sum of v over the
// threads before this one; *total (optional) receives the sum over all threads.  `part` holds n/64 + 1 words of LDS.
__device__ inline uint32_t block_exclusive_scan(uint32_t v, uint32_t *part, uint32_t *total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t t = __shfl_up(inc, off);
    if (lane >= off) inc += t;
  }
  __syncthreads();  // part may still be read from a previous call
  if (lane == 63) part[w] = inc;
  __syncthreads();
  uint32_t base = 0, all = 0;
  for (int i = 0; i < nw; ++i) {
    const uint32_t p = part[i];
    if (i < w) base += p;
    all += p;
  }
  if (total) *total = all;
  return base + inc - v;
}

// Scatter offsets of one radix pass from the digit-major tile histogram hist[digit][tile]: workgroup d turns row d
// into its exclusive prefix over the tiles (in place) and leaves the row total in totals[d] ...
__global__ __launch_bounds__(256) void k_scan_rows(uint32_t *hist, int nTiles, uint32_t *totals) {
  __shared__ uint32_t part[5];
  uint32_t *row = hist + (size_t)blockIdx.x * nTiles;
  uint32_t carry = 0;
  for (int t0 = 0; t0 < nTiles; t0 += 256) {
    const int t = t0 + threadIdx.x;
    const uint32_t v = t < nTiles ? row[t] : 0u;
    uint32_t all;
    const uint32_t ex = block_exclusive_scan(v, part, &all);
    if (t < nTiles) row[t] = carry + ex;
    carry += all;
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}
// ... and one workgroup turns the 256 digit totals into the digits' base offsets.
__global__ __launch_bounds__(256) void k_scan_totals(uint32_t *totals) {
  __shared__ uint32_t part[5];
  const uint32_t v = totals[threadIdx.x];
  const uint32_t ex = block_exclusive_scan(v, part, nullptr);
  totals[threadIdx.x] = ex;
}

// Stable scatter of one 8-bit digit: rank inside the wavefront by ballot matching, wavefronts in order.
__global__ void k_sort_scatter(const uint64_t *__restrict__ kin, const uint32_t *__restrict__ vin,
                               uint64_t *__restrict__ kout, uint32_t *__restrict__ vout, int N, int shift, int nTiles,
                               const uint32_t *__restrict__ offs, const uint32_t *__restrict__ digit_base) {
  __shared__ uint32_t wcnt[SORT_TILE / 64][256];
  for (int w = 0; w < SORT_TILE / 64; ++w) wcnt[w][threadIdx.x] = 0;
  __syncthreads();
  const int i = blockIdx.x * SORT_TILE + threadIdx.x;
  const bool valid = i < N;
  const uint64_t key = valid ? kin[i] : 0ull;
  const uint32_t digit = (uint32_t)(key >> shift) & 255u;
  uint64_t peers = __ballot(valid);
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    const bool bit = (digit >> b) & 1u;
    const uint64_t m = __ballot(bit);
    peers &= bit ? m : ~m;
  }
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const uint32_t rank = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
  if (valid && rank == 0) wcnt[w][digit] = (uint32_t)__popcll(peers);
  __syncthreads();
  if (valid) {
    uint32_t pos = digit_base[digit] + offs[digit * nTiles + blockIdx.x] + rank;
    for (int ww = 0; ww < w; ++ww) pos += wcnt[ww][digit];
    kout[pos] = key;
    vout[pos] = vin[i];
  }
}

struct CsrOut {
  int32_t *perm, *inv_perm, *tok_item, *tok_cmp, *tok_slc, *tok_win;
  int32_t *cmp_start, *slc_start, *win_start, *slc_child_start, *cmp_slc, *cmp_batch, *slc_batch;
};

// Block ids are running counts of block heads (a token whose key prefix differs from its predecessor's) at the three
// granularities.  Three launches: per-tile head counts, their prefix over the tiles (one small workgroup), then every
// tile numbers its own tokens and writes all per-token and per-block arrays.
constexpr int CSR_TILE = 256;
struct Heads { bool c, s, w; };

// Where the blocks begin and which item a sorted position belongs to, for the two kinds of partition.
// Voxel grid: sorted (item << item_shift | Morton) keys; a block of side m is a change of the key above 3*log2(m) bits.
struct GridSrc {
  const uint64_t *ks;
  const uint32_t *vals;  // sorted position -> caller index
  int sc, ss, sw, item_shift;
  __device__ Heads heads(int i) const {
    const uint64_t k = ks[i], p = i == 0 ? 0ull : ks[i - 1];
    const bool first = i == 0;
    return Heads{first || (k >> sc) != (p >> sc), first || (k >> ss) != (p >> ss), first || (k >> sw) != (p >> sw)};
  }
  __device__ int item(int i) const { return (int)(ks[i] >> item_shift); }
  __device__ int32_t source(int i) const { return (int32_t)vals[i]; }
};
// Sequences: the caller's order is the token order; blocks are runs of lc / ls / lw tokens counted from the start of
// each sequence (the last one of a sequence may be shorter).
struct SeqSrc {
  const int32_t *offs;
  int B, lc, ls, lw;
  __device__ int item(int i) const {
    int lo = 0, hi = B;  // offs[lo] <= i < offs[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (offs[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
  }
  __device__ Heads heads(int i) const {
    const int pos = i - offs[item(i)];
    return Heads{pos % lc == 0, pos % ls == 0, pos % lw == 0};
  }
  __device__ int32_t source(int i) const { return i; }
};

template <class Src>
__global__ __launch_bounds__(CSR_TILE) void k_csr_count(Src src, int N, int nTiles, uint32_t *__restrict__ tile_cnt) {
  __shared__ uint32_t cnt[3];
  if (threadIdx.x < 3) cnt[threadIdx.x] = 0;
  __syncthreads();
  const int i = blockIdx.x * CSR_TILE + threadIdx.x;
  Heads h{false, false, false};
  if (i < N) h = src.heads(i);
  const uint64_t bc = __ballot(h.c), bs = __ballot(h.s), bw = __ballot(h.w);
  if ((threadIdx.x & 63) == 0) {
    atomicAdd(&cnt[0], (uint32_t)__popcll(bc));
    atomicAdd(&cnt[1], (uint32_t)__popcll(bs));
    atomicAdd(&cnt[2], (uint32_t)__popcll(bw));
  }
  __syncthreads();
  if (threadIdx.x < 3) tile_cnt[threadIdx.x * nTiles + blockIdx.x] = cnt[threadIdx.x];
}

// Exclusive prefix of the three count rows over the tiles (in place); one workgroup.
__global__ __launch_bounds__(256) void k_csr_scan(uint32_t *tile_cnt, int nTiles) {
  __shared__ uint32_t part[5];
  for (int x = 0; x < 3; ++x) {
    uint32_t *row = tile_cnt + (size_t)x * nTiles;
    uint32_t carry = 0;
    for (int t0 = 0; t0 < nTiles; t0 += 256) {
      const int t = t0 + threadIdx.x;
      const uint32_t v = t < nTiles ? row[t] : 0u;
      uint32_t all;
      const uint32_t ex = block_exclusive_scan(v, part, &all);
      if (t < nTiles) row[t] = carry + ex;
      carry += all;
    }
  }
}

template <class Src>
__global__ __launch_bounds__(CSR_TILE) void k_csr_write(Src src, int N, int B, int nTiles,
                                                        const uint32_t *__restrict__ tile_base, CsrOut o, int32_t *meta) {
  __shared__ uint32_t part[5];
  const int i = blockIdx.x * CSR_TILE + threadIdx.x;
  Heads h{false, false, false};
  if (i < N) h = src.heads(i);
  // inclusive head counts up to and including token i
  const int idc = (int)(tile_base[blockIdx.x] + block_exclusive_scan(h.c, part, nullptr) + h.c) - 1;
  const int ids = (int)(tile_base[nTiles + blockIdx.x] + block_exclusive_scan(h.s, part, nullptr) + h.s) - 1;
  const int idw = (int)(tile_base[2 * nTiles + blockIdx.x] + block_exclusive_scan(h.w, part, nullptr) + h.w) - 1;
  if (i >= N) return;
  const int item = src.item(i);
  const int pitem = i == 0 ? -1 : src.item(i - 1);
  const int32_t from = src.source(i);
  o.perm[i] = from;
  o.inv_perm[from] = i;
  o.tok_item[i] = item;
  o.tok_cmp[i] = idc;
  o.tok_slc[i] = ids;
  o.tok_win[i] = idw;
  if (h.c) { o.cmp_start[idc] = i; o.cmp_slc[idc] = ids; }
  if (h.s) { o.slc_start[ids] = i; o.slc_child_start[ids] = idc; }
  if (h.w) o.win_start[idw] = i;
  for (int it = pitem + 1; it <= item; ++it) { o.cmp_batch[it] = idc; o.slc_batch[it] = ids; }
  if (i == N - 1) {
    const int Nc = idc + 1, Ns = ids + 1, Nw = idw + 1;
    o.cmp_start[Nc] = N; o.slc_start[Ns] = N; o.win_start[Nw] = N; o.slc_child_start[Ns] = Nc;
    for (int it = item + 1; it <= B; ++it) { o.cmp_batch[it] = Nc; o.slc_batch[it] = Ns; }
    meta[META_NC] = Nc; meta[META_NS] = Ns; meta[META_NW] = Nw;
  }
}

// Validation of the batch offsets alone (the sequence builder has no coordinates to read).
__global__ void k_check_offsets(const int32_t *__restrict__ offs, int N, int B, int32_t *meta) {
  for (int j = blockIdx.x * blockDim.x + threadIdx.x; j <= B; j += gridDim.x * blockDim.x) {
    const int o = offs[j];
    const bool bad = (j == 0 && o != 0) || (j == B && o != N) || (j > 0 && o < offs[j - 1]) || o < 0 || o > N;
    if (bad) atomicOr(&meta[META_ERR], 1);
  }
}

// Largest per-item block counts and per-block token counts (integer max: order independent).
__global__ void k_maxima(CsrOut o, int B, int32_t *meta) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int Nc = meta[META_NC], Ns = meta[META_NS], Nw = meta[META_NW];
  if (i < B) {
    atomicMax(&meta[META_SMAX], o.slc_batch[i + 1] - o.slc_batch[i]);
    atomicMax(&meta[META_CMAX], o.cmp_batch[i + 1] - o.cmp_batch[i]);
  }
  if (i < Nc) atomicMax(&meta[META_CMP_TOK], o.cmp_start[i + 1] - o.cmp_start[i]);
  if (i < Ns) atomicMax(&meta[META_SLC_TOK], o.slc_start[i + 1] - o.slc_start[i]);
  if (i < Nw) atomicMax(&meta[META_WIN_TOK], o.win_start[i + 1] - o.win_start[i]);
}

}  // namespace

// Stable LSD radix sort of n (key, value) pairs by the low `bits` bits of the keys, 8 bits per pass, ping-ponging between
// (k0, v0) and (k1, v1); `aux` holds sort_pairs_aux_bytes(n) bytes.  Returns 0 when the sorted pairs end in (k0, v0),
// 1 when they end in (k1, v1).  Four launches per pass on `stream`, no allocation, no synchronisation.
size_t sort_pairs_aux_bytes(int n) {
  const int nTiles = (n + SORT_TILE - 1) / SORT_TILE;
  return align_up((size_t)256 * (nTiles > 0 ? nTiles : 1) * 4, 256) + 256 * 4;
}
int sort_pairs(uint64_t *k0, uint32_t *v0, uint64_t *k1, uint32_t *v1, void *aux, int n, int bits, hipStream_t stream) {
  const int nTiles = (n + SORT_TILE - 1) / SORT_TILE;
  uint32_t *hist = (uint32_t *)aux;
  uint32_t *digit_base = (uint32_t *)((char *)aux + align_up((size_t)256 * (nTiles > 0 ? nTiles : 1) * 4, 256));
  int where = 0;
  if (n <= 0) return where;
  for (int shift = 0; shift < bits; shift += 8) {
    k_sort_hist<<<nTiles, SORT_TILE, 0, stream>>>(k0, n, shift, nTiles, hist);
    k_scan_rows<<<256, 256, 0, stream>>>(hist, nTiles, digit_base);
    k_scan_totals<<<1, 256, 0, stream>>>(digit_base);
    k_sort_scatter<<<nTiles, SORT_TILE, 0, stream>>>(k0, v0, k1, v1, n, shift, nTiles, hist, digit_base);
    uint64_t *tk = k0; k0 = k1; k1 = tk;
    uint32_t *tv = v0; v0 = v1; v1 = tv;
    where ^= 1;
  }
  return where;
}

// Common part of the two builders: grid_mode = voxel partition (sort by Morton key), else sequences in caller order.
static int build_handle(const ssa_params_t *p, const int32_t *coords, const int32_t *batch_offsets, bool grid_mode,
                        hipStream_t stream, ssa_blocks_t **out) {
  const int N = p->n_tokens, B = p->n_batch;
  int bits = 1;
  while ((1 << bits) < p->grid) ++bits;
  int item_bits = 1;
  while ((1ll << item_bits) < (long long)B) ++item_bits;

  ssa_blocks *h = new ssa_blocks();
  h->N = N; h->B = B; h->G = p->grid; h->m_cmp = p->m_cmp; h->m_slc = p->m_slc; h->m_win = p->m_win;
  h->bits = grid_mode ? bits : 0;
  h->dims = grid_mode ? 3 : 1;
  if (hipGetDevice(&h->device) != hipSuccess) { delete h; return SSA_ERR_HIP; }
  const size_t n1 = (size_t)N + 1;
  const size_t ints = 2 * (size_t)N + 6 * (size_t)N + 4 * n1 + (size_t)N + 3 * ((size_t)B + 1) + 64;
  if (hipMalloc(&h->base, ints * sizeof(int32_t)) != hipSuccess) { delete h; return SSA_ERR_HIP; }
  int32_t *w = (int32_t *)h->base;
  auto take = [&](size_t n) { int32_t *r = w; w += n; return r; };
  h->sorted_keys = (uint64_t *)take(2 * (size_t)N);  // first: the allocation's alignment serves the 8-byte keys
  h->perm = take(N); h->inv_perm = take(N); h->tok_item = take(N); h->tok_cmp = take(N); h->tok_slc = take(N);
  h->tok_win = take(N); h->cmp_start = take(n1); h->slc_start = take(n1); h->win_start = take(n1);
  h->slc_child_start = take(n1); h->cmp_slc = take(N); h->cmp_batch = take(B + 1); h->slc_batch = take(B + 1);
  h->item_start = take(B + 1);

  int32_t meta_h[META_N] = {0};
  const int nTiles = (N + SORT_TILE - 1) / SORT_TILE;
  void *tmp = nullptr;
  const size_t key_b = align_up((size_t)N * 8, 256), val_b = align_up((size_t)N * 4, 256);
  const size_t hist_b = align_up((size_t)256 * (nTiles > 0 ? nTiles : 1) * 4, 256);
  const int csrTiles = (N + CSR_TILE - 1) / CSR_TILE;
  const size_t aux_b = align_up((size_t)(256 + 3 * (csrTiles > 0 ? csrTiles : 1)) * 4, 256);  // digit bases | CSR tile counts
  const size_t tmp_bytes = (grid_mode ? 2 * key_b + 2 * val_b + hist_b : 0) + aux_b + 256;
  auto fail = [&](int code) {
    if (tmp) (void)hipFree(tmp);
    (void)hipFree(h->base);
    delete h;
    return code;
  };
  if (hipMalloc(&tmp, tmp_bytes) != hipSuccess) return fail(SSA_ERR_HIP);
  char *tp = (char *)tmp;
  uint64_t *k0 = nullptr, *k1 = nullptr;
  uint32_t *v0 = nullptr, *v1 = nullptr, *hist = nullptr;
  if (grid_mode) {
    k0 = (uint64_t *)tp; tp += key_b;
    k1 = (uint64_t *)tp; tp += key_b;
    v0 = (uint32_t *)tp; tp += val_b;
    v1 = (uint32_t *)tp; tp += val_b;
    hist = (uint32_t *)tp; tp += hist_b;
  }
  uint32_t *digit_base = (uint32_t *)tp, *tile_cnt = digit_base + 256; tp += aux_b;
  int32_t *meta = (int32_t *)tp;
  if (hipMemsetAsync(meta, 0, 256, stream) != hipSuccess) return fail(SSA_ERR_HIP);
  CsrOut o{h->perm, h->inv_perm, h->tok_item, h->tok_cmp, h->tok_slc, h->tok_win, h->cmp_start, h->slc_start,
           h->win_start, h->slc_child_start, h->cmp_slc, h->cmp_batch, h->slc_batch};
  if (N == 0) {
    // no tokens: every start array is a single zero; the offsets are still validated (all must be zero)
    if (hipMemsetAsync(h->base, 0, ints * sizeof(int32_t), stream) != hipSuccess) return fail(SSA_ERR_HIP);
    k_check_offsets<<<1, 256, 0, stream>>>(batch_offsets, 0, B, meta);
  } else if (grid_mode) {
    k_make_keys<<<(N + 255) / 256, 256, 0, stream>>>(coords, batch_offsets, N, B, p->grid, bits, k0, v0, meta);
    const int total_bits = 3 * bits + item_bits;
    for (int shift = 0; shift < total_bits; shift += 8) {
      k_sort_hist<<<nTiles, SORT_TILE, 0, stream>>>(k0, N, shift, nTiles, hist);
      k_scan_rows<<<256, 256, 0, stream>>>(hist, nTiles, digit_base);
      k_scan_totals<<<1, 256, 0, stream>>>(digit_base);
      k_sort_scatter<<<nTiles, SORT_TILE, 0, stream>>>(k0, v0, k1, v1, N, shift, nTiles, hist, digit_base);
      uint64_t *tk = k0; k0 = k1; k1 = tk;
      uint32_t *tv = v0; v0 = v1; v1 = tv;
    }
    const GridSrc src{k0, v0, 3 * ilog2_exact(p->m_cmp), 3 * ilog2_exact(p->m_slc), 3 * ilog2_exact(p->m_win), 3 * bits};
    k_csr_count<<<csrTiles, CSR_TILE, 0, stream>>>(src, N, csrTiles, tile_cnt);
    k_csr_scan<<<1, 256, 0, stream>>>(tile_cnt, csrTiles);
    k_csr_write<<<csrTiles, CSR_TILE, 0, stream>>>(src, N, B, csrTiles, tile_cnt, o, meta);
    if (hipMemcpyAsync(h->sorted_keys, k0, (size_t)N * sizeof(uint64_t), hipMemcpyDeviceToDevice, stream) != hipSuccess)
      return fail(SSA_ERR_HIP);
  } else {
    // The offsets are checked first and the result is read back before any kernel searches them: SeqSrc::item assumes
    // ascending offsets that start at 0 and end at N.
    k_check_offsets<<<1, 256, 0, stream>>>(batch_offsets, N, B, meta);
    if (hipMemcpyAsync(meta_h, meta, sizeof(meta_h), hipMemcpyDeviceToHost, stream) != hipSuccess) return fail(SSA_ERR_HIP);
    if (hipStreamSynchronize(stream) != hipSuccess) return fail(SSA_ERR_HIP);
    if (meta_h[META_ERR] & 1) return fail(SSA_ERR_BAD_OFFSETS);
    const SeqSrc src{batch_offsets, B, p->m_cmp, p->m_slc, p->m_win};
    k_csr_count<<<csrTiles, CSR_TILE, 0, stream>>>(src, N, csrTiles, tile_cnt);
    k_csr_scan<<<1, 256, 0, stream>>>(tile_cnt, csrTiles);
    k_csr_write<<<csrTiles, CSR_TILE, 0, stream>>>(src, N, B, csrTiles, tile_cnt, o, meta);
    if (hipMemsetAsync(h->sorted_keys, 0, (size_t)N * sizeof(uint64_t), stream) != hipSuccess) return fail(SSA_ERR_HIP);
  }
  if (N > 0) {
    const int span = (N > B ? N : B);
    k_maxima<<<(span + 255) / 256, 256, 0, stream>>>(o, B, meta);
  }
  if (hipMemcpyAsync(h->item_start, batch_offsets, ((size_t)B + 1) * sizeof(int32_t), hipMemcpyDeviceToDevice, stream) !=
      hipSuccess)
    return fail(SSA_ERR_HIP);
  if (hipGetLastError() != hipSuccess) return fail(SSA_ERR_HIP);
  if (hipMemcpyAsync(meta_h, meta, sizeof(meta_h), hipMemcpyDeviceToHost, stream) != hipSuccess) return fail(SSA_ERR_HIP);
  if (hipStreamSynchronize(stream) != hipSuccess) return fail(SSA_ERR_HIP);
  if (meta_h[META_ERR] & 1) return fail(SSA_ERR_BAD_OFFSETS);
  if (meta_h[META_ERR] & 2) return fail(SSA_ERR_COORD_RANGE);
  (void)hipFree(tmp);
  tmp = nullptr;
  h->Nc = meta_h[META_NC]; h->Ns = meta_h[META_NS]; h->Nw = meta_h[META_NW];
  h->s_max = meta_h[META_SMAX]; h->c_max = meta_h[META_CMAX]; h->slc_tok_max = meta_h[META_SLC_TOK];
  h->win_tok_max = meta_h[META_WIN_TOK]; h->cmp_tok_max = meta_h[META_CMP_TOK];
  *out = h;
  return SSA_OK;
}

extern "C" int ssa_build_blocks(const ssa_params_t *p, const int32_t *coords, const int32_t *batch_offsets,
                                void *stream_, ssa_blocks_t **out) {
  if (!p || !out) return SSA_ERR_NULL;
  *out = nullptr;
  if (p->n_tokens < 0 || p->n_batch < 1 || p->grid < 1 || p->grid > 1024) return SSA_ERR_BAD_SHAPE;
  if (p->m_cmp < 1 || p->m_slc < 1 || p->m_win < 1 || p->m_slc <= p->m_cmp || p->m_slc % p->m_cmp != 0)
    return SSA_ERR_BAD_BLOCK_SIZES;
  auto pow2 = [](int m) { return (m & (m - 1)) == 0; };
  if (!pow2(p->m_cmp) || !pow2(p->m_slc) || !pow2(p->m_win)) return SSA_ERR_UNSUPPORTED;
  if (!batch_offsets || (p->n_tokens > 0 && !coords)) return SSA_ERR_NULL;
  return build_handle(p, coords, batch_offsets, true, (hipStream_t)stream_, out);
}

extern "C" int ssa_build_blocks_1d(const ssa_params_t *p, const int32_t *batch_offsets, void *stream_,
                                   ssa_blocks_t **out) {
  if (!p || !out) return SSA_ERR_NULL;
  *out = nullptr;
  if (p->n_tokens < 0 || p->n_batch < 1) return SSA_ERR_BAD_SHAPE;
  if (p->m_cmp < 1 || p->m_slc < 1 || p->m_win < 1 || p->m_slc <= p->m_cmp || p->m_slc % p->m_cmp != 0)
    return SSA_ERR_BAD_BLOCK_SIZES;
  if (!batch_offsets) return SSA_ERR_NULL;
  return build_handle(p, nullptr, batch_offsets, false, (hipStream_t)stream_, out);
}

extern "C" int ssa_blocks_counts(const ssa_blocks_t *b, int32_t *n_cmp, int32_t *n_slc, int32_t *n_win) {
  if (!b) return SSA_ERR_NULL;
  if (n_cmp) *n_cmp = b->Nc;
  if (n_slc) *n_slc = b->Ns;
  if (n_win) *n_win = b->Nw;
  return SSA_OK;
}

extern "C" int ssa_blocks_max_slc_per_item(const ssa_blocks_t *b, int32_t *s_max) {
  if (!b || !s_max) return SSA_ERR_NULL;
  *s_max = b->s_max;
  return SSA_OK;
}

extern "C" int ssa_blocks_export(const ssa_blocks_t *b, int which, void *dst, size_t bytes, void *stream) {
  if (!b || !dst) return SSA_ERR_NULL;
  const int32_t *src = nullptr;
  size_t n = 0;
  switch (which) {
    case SSA_ARR_PERM: src = b->perm; n = b->N; break;
    case SSA_ARR_INV_PERM: src = b->inv_perm; n = b->N; break;
    case SSA_ARR_CMP_START: src = b->cmp_start; n = (size_t)b->Nc + 1; break;
    case SSA_ARR_SLC_START: src = b->slc_start; n = (size_t)b->Ns + 1; break;
    case SSA_ARR_WIN_START: src = b->win_start; n = (size_t)b->Nw + 1; break;
    case SSA_ARR_SLC_CHILD_START: src = b->slc_child_start; n = (size_t)b->Ns + 1; break;
    case SSA_ARR_CMP_BATCH: src = b->cmp_batch; n = (size_t)b->B + 1; break;
    case SSA_ARR_SLC_BATCH: src = b->slc_batch; n = (size_t)b->B + 1; break;
    case SSA_ARR_TOK_WIN: src = b->tok_win; n = b->N; break;
    default: return SSA_ERR_BAD_SHAPE;
  }
  if (bytes < n * sizeof(int32_t)) return SSA_ERR_WORKSPACE;
  if (n == 0) return SSA_OK;
  SSA_HIP_TRY(hipMemcpyAsync(dst, src, n * sizeof(int32_t), hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return SSA_OK;
}

extern "C" void ssa_blocks_destroy(ssa_blocks_t *b) {
  if (!b) return;
  if (b->base) (void)hipFree(b->base);
  delete b;
}
