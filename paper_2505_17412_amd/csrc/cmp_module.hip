// Learned sparse 3D compression module for gfx950: x + PE, sparse 3x3x3 convolution, mean pool (paper, Sec. "Sparse 3D
// Compression", eq. (5)), forward and backward.
//
// Readings (the paper gives the three operations and nothing else): PE is a table [m_cmp^3][C] indexed by the
// token's place inside its compression block, row ((x mod m)*m + (y mod m))*m + (z mod m); the convolution is a
// submanifold 3x3x3 one over the sparse volume of the token's batch item (outputs at active sites, inactive
// neighbours contribute nothing), C -> C channels with bias, C = H_kv * head_dim; w[o] is [C_in][C_out] for
// offset o = ((dx+1)*3 + (dy+1))*3 + (dz+1) and multiplies the token at coords + (dx,dy,dz); the mean runs over
// the active tokens of the compression block.  Coordinates must be distinct inside an item.
//
// Layout: everything is done in the sorted (Morton) token order of the block structure.  The neighbour of a
// token is found by binary search of its Morton key among the sorted keys the handle keeps.  The convolution is a
// gather-GEMM on the matrix cores: a wavefront owns 64 tokens (four 16-row MFMA tiles) and 32 output channels,
// and for each of the 27 offsets multiplies the gathered neighbour rows (A operand, 16 bytes per lane straight
// from memory) with the offset's C x C weights (B operand, contraction index contiguous).  The data gradient is
// the same kernel on mirrored offsets with the weights read the other way round; the weight gradient contracts
// over tokens, its two operands come from row-major LDS tiles through the transposing LDS read.  No floating
// point atomics anywhere: partial sums are written per chunk and added in a fixed order.
#include "mfma_common.h"
#include "mfma_qc.h"
#include "profile.h"

namespace {

__device__ inline uint32_t compact3(uint64_t v64) {  // bits 0,3,6,.. of v -> bits 0,1,2,..
  uint32_t v = (uint32_t)v64 & 0x09249249u;
  v = (v | (v >> 2)) & 0x030C30C3u;
  v = (v | (v >> 4)) & 0x0300F00Fu;
  v = (v | (v >> 8)) & 0x030000FFu;
  v = (v | (v >> 16)) & 0x3FFu;
  return v;
}
__device__ inline uint32_t spread3m(uint32_t v) {
  v &= 0x3FFu;
  v = (v | (v << 16)) & 0x030000FFu;
  v = (v | (v << 8)) & 0x0300F00Fu;
  v = (v | (v << 4)) & 0x030C30C3u;
  v = (v | (v << 2)) & 0x09249249u;
  return v;
}
struct Site { int item, x, y, z; };
__device__ inline Site decode(uint64_t key, int bits) {
  const uint64_t code = key & ((1ull << (3 * bits)) - 1ull);
  return Site{(int)(key >> (3 * bits)), (int)compact3(code >> 2), (int)compact3(code >> 1), (int)compact3(code)};
}

// nbr[pos][o] = sorted position of the token at coords(pos) + offset o in the same item, or -1.  One thread per
// (pos, o): a binary search of the neighbour's key inside the item's range of the sorted keys.
__global__ void c_neighbors(const uint64_t *__restrict__ keys, const int32_t *__restrict__ item_start, int N, int G,
                            int bits, int32_t *__restrict__ nbr) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)N * 27) return;
  const int pos = (int)(i / 27), o = (int)(i % 27);
  const Site s = decode(keys[pos], bits);
  const int x = s.x + o / 9 - 1, y = s.y + o / 3 % 3 - 1, z = s.z + o % 3 - 1;
  int found = -1;
  if ((unsigned)x < (unsigned)G && (unsigned)y < (unsigned)G && (unsigned)z < (unsigned)G) {
    const uint64_t want = ((uint64_t)s.item << (3 * bits)) |
                          (uint64_t)((spread3m((uint32_t)x) << 2) | (spread3m((uint32_t)y) << 1) | spread3m((uint32_t)z));
    int lo = item_start[s.item];
    const int e = item_start[s.item + 1];
    int hi = e;  // first position in [lo, e) whose key is >= want
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (keys[mid] < want) lo = mid + 1; else hi = mid;
    }
    if (lo < e && keys[lo] == want) found = lo;
  }
  nbr[i] = found;
}

// U[pos] = x[perm[pos]] + PE[place of the token inside its block]   (bf16, sorted order)
__global__ void c_add_pe(const bf16_t *__restrict__ x, const bf16_t *__restrict__ pe, const int32_t *__restrict__ perm,
                         const uint64_t *__restrict__ keys, int N, int C, int bits, int m, bf16_t *__restrict__ U) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per = C / 8;
  if (i >= (size_t)N * per) return;
  const int pos = (int)(i / per), c0 = (int)(i % per) * 8;
  const Site s = decode(keys[pos], bits);
  const int p = ((s.x & (m - 1)) * m + (s.y & (m - 1))) * m + (s.z & (m - 1));
  const bf16x8 a = ld8(x + (size_t)perm[pos] * C + c0), b = ld8(pe + (size_t)p * C + c0);
  bf16x8 r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r[j] = (__bf16)((float)a[j] + (float)b[j]);
  *reinterpret_cast<bf16x8 *>(U + (size_t)pos * C + c0) = r;
}

// Wt[o][c_out][c_in] = w[o][c_in][c_out]
__global__ void c_transpose_w(const bf16_t *__restrict__ w, int C, bf16_t *__restrict__ wt) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)27 * C * C) return;
  const int ci = (int)(i % C), co = (int)(i / C % C), o = (int)(i / ((size_t)C * C));
  wt[i] = w[((size_t)o * C + ci) * C + co];
}

// Gather-GEMM: out[pos][n] = bias[n] + sum_o sum_k in[nbr[pos][o']][k] * Bw[o][n][k], o' = o (forward) or 26 - o
// (data gradient: the token that took `pos` as its neighbour o sits at the mirrored offset).  Bw holds, per offset,
// a [C][C] matrix with the contraction index contiguous.
template <int C, bool MIRROR, int MT, int NBW>
__global__ __launch_bounds__(256) void c_conv(const bf16_t *__restrict__ in, const int32_t *__restrict__ nbr,
                                              const bf16_t *__restrict__ Bw, const bf16_t *__restrict__ bias, int N,
                                              float *__restrict__ out) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int pos0 = (blockIdx.x * 4 + wid) * 16 * MT;  // a wavefront owns MT tiles of 16 tokens: every weight operand
  if (pos0 >= N) return;                               // it loads feeds MT matrix instructions
  const int nb0 = blockIdx.y * NBW;                    // blockIdx.y: which NBW blocks of 16 output channels
  f32x4 acc[MT][NBW];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) acc[a][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  int tok[MT], nxt[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    tok[a] = pos0 + 16 * a + n;
    nxt[a] = tok[a] < N ? nbr[(size_t)tok[a] * 27 + (MIRROR ? 26 : 0)] : -1;
  }
  for (int o = 0; o < 27; ++o) {
    // the neighbour indices of the next offset are requested before this offset's rows are used: the two dependent
    // loads (index, then row) of consecutive offsets overlap
    int src[MT];
    bool some = false;
#pragma unroll
    for (int a = 0; a < MT; ++a) {
      src[a] = nxt[a];
      some = some || src[a] >= 0;
      if (o + 1 < 27) nxt[a] = tok[a] < N ? nbr[(size_t)tok[a] * 27 + (MIRROR ? 25 - o : o + 1)] : -1;
    }
    if (!__any(some)) continue;
    const bf16_t *Bo = Bw + (size_t)o * C * C;
#pragma unroll
    for (int ks = 0; ks < C / 32; ++ks) {
      bf16x8 av[MT];
#pragma unroll
      for (int a = 0; a < MT; ++a) av[a] = src[a] >= 0 ? ld8(in + (size_t)src[a] * C + 32 * ks + 8 * quad) : zero8();
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb) {
        const bf16x8 bv = ld8(Bo + (size_t)(16 * (nb0 + nb) + n) * C + 32 * ks + 8 * quad);
#pragma unroll
        for (int a = 0; a < MT; ++a) acc[a][nb] = mfma16(av[a], bv, acc[a][nb]);
      }
    }
  }
  // C layout: lane holds output channel 16*(nb0 + nb) + n of tokens pos0 + 16*a + 4*quad + i
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb) {
    const int ch = 16 * (nb0 + nb) + n;
    const float bs = bias ? bf16_to_f32(bias[ch]) : 0.f;
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = pos0 + 16 * a + 4 * quad + i;
        if (t < N) out[(size_t)t * C + ch] = acc[a][nb][i] + bs;
      }
  }
}

// The same gather-GEMM for C = 128 with both operands staged through LDS: a workgroup owns TOK tokens, wavefront w the
// output channels 32w .. 32w+31.  Per offset the 128 x 128 weights (32 KB) and the TOK gathered rows are written to LDS
// once and read by all four wavefronts as conflict-free row-operand reads; the data of the next offset is in flight in
// registers meanwhile, its row indices taken from a copy of the tile's neighbour table in LDS.  Row r of a 16-row MFMA
// tile stands for LDS row 8*(r >> 2) + 4*a + (r & 3) of its 32-row tile (a = which half), for tokens and for channels
// alike; the store at the end undoes that numbering.
constexpr int CONV_TOK = 128;  // tokens per workgroup of the staged convolution
template <bool MIRROR, int TOK>
__global__ __launch_bounds__(256) void c_conv128(const bf16_t *__restrict__ in, const int32_t *__restrict__ nbr,
                                                 const bf16_t *__restrict__ Bw, const bf16_t *__restrict__ bias, int N,
                                                 float *__restrict__ out) {
  constexpr int C = 128, MT = TOK / 16, AI = TOK / 16;  // AI: gathered 16-byte items per thread (TOK x 16 / 256)
  using G = TileGeom<C>;
  __shared__ __align__(16) bf16_t sw[4 * G::ROW_ELEMS], sa[(TOK / 32) * G::ROW_ELEMS];
  __shared__ int any_flag[27];
  __shared__ int32_t snbr[TOK * 27];
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  const int pos0 = blockIdx.x * TOK;
  // which offsets have a neighbour for any of the tokens (workgroup-uniform skip)
  if (threadIdx.x < 27) any_flag[threadIdx.x] = 0;
  __syncthreads();
  for (int i = threadIdx.x; i < TOK * 27; i += 256) {
    const int t = pos0 + i / 27, o = i % 27;
    const int32_t v = t < N ? nbr[(size_t)t * 27 + o] : -1;
    snbr[i] = v;
    if (v >= 0) any_flag[MIRROR ? 26 - o : o] = 1;
  }
  __syncthreads();
  f32x4 acc[MT][2];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt][0] = acc[mt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
  // staging roles: the weights are 128 rows x 16 segments = 2048 items (8 per thread), the gathered rows TOK x 16
  bf16x8 rw[8], ra[AI];
  auto fetch = [&](int o) {
    const bf16_t *Bo = Bw + (size_t)o * C * C;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int it = threadIdx.x + 256 * i;
      rw[i] = ld8(Bo + (size_t)(it / 16) * C + 8 * (it % 16));
    }
    const int oo = MIRROR ? 26 - o : o;
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int it = threadIdx.x + 256 * i;
      const int src = snbr[(it / 16) * 27 + oo];
      ra[i] = src >= 0 ? ld8(in + (size_t)src * C + 8 * (it % 16)) : zero8();
    }
  };
  int o = 0;
  while (o < 27 && !any_flag[o]) ++o;
  if (o < 27) fetch(o);
  while (o < 27) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int it = threadIdx.x + 256 * i, row = it / 16;
      *reinterpret_cast<bf16x8 *>(sw + (row >> 5) * G::ROW_ELEMS + G::row_off(row & 31, it % 16)) = rw[i];
    }
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int it = threadIdx.x + 256 * i, row = it / 16;
      *reinterpret_cast<bf16x8 *>(sa + (row >> 5) * G::ROW_ELEMS + G::row_off(row & 31, it % 16)) = ra[i];
    }
    __syncthreads();
    int nxt = o + 1;
    while (nxt < 27 && !any_flag[nxt]) ++nxt;
    if (nxt < 27) fetch(nxt);
#pragma unroll
    for (int ks = 0; ks < C / 32; ++ks) {
      const bf16x8 b0 = lds_row_operand<C>(sw + wid * G::ROW_ELEMS, 0, ks), b1 = lds_row_operand<C>(sw + wid * G::ROW_ELEMS, 1, ks);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const bf16x8 av = lds_row_operand<C>(sa + (mt >> 1) * G::ROW_ELEMS, mt & 1, ks);
        acc[mt][0] = mfma16(av, b0, acc[mt][0]);
        acc[mt][1] = mfma16(av, b1, acc[mt][1]);
      }
    }
    __syncthreads();
    o = nxt;
  }
  // lane: column n of half a -> channel 32*wid + 8*(n >> 2) + 4*a + (n & 3); rows 4*quad + i of tile mt -> token
  // pos0 + 32*(mt >> 1) + 8*quad + 4*(mt & 1) + i
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int ch = 32 * wid + 8 * (n >> 2) + 4 * a + (n & 3);
    const float bs = bias ? bf16_to_f32(bias[ch]) : 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = pos0 + 32 * (mt >> 1) + 8 * quad + 4 * (mt & 1) + i;
        if (t < N) out[(size_t)t * C + ch] = acc[mt][a][i] + bs;
      }
  }
}

// Mean over the tokens of each compression block (contiguous in sorted order); one workgroup per block.
__global__ void c_pool(const float *__restrict__ Y, const int32_t *__restrict__ cmp_start, int C, bf16_t *__restrict__ xc) {
  const int c = blockIdx.x, b = cmp_start[c], e = cmp_start[c + 1];
  const float inv = 1.0f / (float)(e - b);  // same arithmetic as the plain mean pool of the attention path
  for (int f = threadIdx.x; f < C; f += blockDim.x) {
    float s = 0.f;
    for (int pos = b; pos < e; ++pos) s += Y[(size_t)pos * C + f];
    xc[(size_t)c * C + f] = f32_to_bf16(s * inv);
  }
}

// dY[pos] = dXc[block(pos)] / count(block)   (bf16, sorted order): gradient of the mean pool
__global__ void c_expand(const float *__restrict__ dxc, const int32_t *__restrict__ tok_cmp,
                         const int32_t *__restrict__ cmp_start, int N, int C, bf16_t *__restrict__ dY) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per = C / 8;
  if (i >= (size_t)N * per) return;
  const int pos = (int)(i / per), c0 = (int)(i % per) * 8;
  const int c = tok_cmp[pos];
  const float inv = 1.0f / (float)(cmp_start[c + 1] - cmp_start[c]);
  bf16x8 r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r[j] = (__bf16)(dxc[(size_t)c * C + c0 + j] * inv);
  *reinterpret_cast<bf16x8 *>(dY + (size_t)pos * C + c0) = r;
}

// dbias[f] = sum over blocks of dXc[c][f]  (the pool's 1/count and the block's count cancel): partial sums over
// DBIAS_PARTS row ranges, added in order by c_sum_parts.
constexpr int DBIAS_PARTS = 32;
__global__ void c_dbias_partial(const float *__restrict__ dxc, int Nc, int C, float *__restrict__ part) {
  const int f = blockIdx.x * blockDim.x + threadIdx.x;
  if (f >= C) return;
  const int per = (Nc + DBIAS_PARTS - 1) / DBIAS_PARTS;
  const int b = min(Nc, (int)blockIdx.y * per), e = min(Nc, b + per);
  float s = 0.f;
  for (int c = b; c < e; ++c) s += dxc[(size_t)c * C + f];
  part[(size_t)blockIdx.y * C + f] = s;
}

// dx[perm[pos]] += dU[pos]   (caller order, parameter dtype)
__global__ void c_dx_accum(const float *__restrict__ dU, const int32_t *__restrict__ perm, int N, int C, bf16_t *dx) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per = C / 8;
  if (i >= (size_t)N * per) return;
  const int pos = (int)(i / per), c0 = (int)(i % per) * 8;
  bf16_t *d = dx + (size_t)perm[pos] * C + c0;
  const bf16x8 cur = ld8(d);
  bf16x8 r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r[j] = (__bf16)((float)cur[j] + dU[(size_t)pos * C + c0 + j]);
  *reinterpret_cast<bf16x8 *>(d) = r;
}

// dPE, first stage: the tokens of chunk blockIdx.x are visited in order, thread f owns channel f of every table row
// (LDS [m^3][C] fp32), so no two threads ever add to the same cell.
__global__ void c_dpe_partial(const float *__restrict__ dU, const uint64_t *__restrict__ keys, int N, int C, int bits, int m,
                              int chunk, float *__restrict__ part) {
  extern __shared__ float tbl[];
  const int rows = m * m * m;
  for (int i = threadIdx.x; i < rows * C; i += blockDim.x) tbl[i] = 0.f;
  __syncthreads();
  const int b = blockIdx.x * chunk, e = min(N, b + chunk);
  for (int pos = b; pos < e; ++pos) {
    const Site s = decode(keys[pos], bits);
    const int p = ((s.x & (m - 1)) * m + (s.y & (m - 1))) * m + (s.z & (m - 1));
    for (int f = threadIdx.x; f < C; f += blockDim.x) tbl[p * C + f] += dU[(size_t)pos * C + f];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < rows * C; i += blockDim.x) part[(size_t)blockIdx.x * rows * C + i] = tbl[i];
}

// Ordered sum of partial results: out[g][i] = sum of part[g*group + j][i], j = 0 .. group-1 (parts past n_parts are
// skipped).  One launch with group = n_parts gives the total; two launches (group, then the group results) keep
// the work parallel when there are many parts.  The order of the additions is fixed either way.
__global__ void c_sum_parts(const float *__restrict__ part, int n_parts, int n_groups, size_t len, float *__restrict__ out) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= len) return;
  const int group = (n_parts + n_groups - 1) / n_groups;
  const int g = blockIdx.y, b = g * group, e = min(n_parts, b + group);
  float s = 0.f;
  for (int k = b; k < e; ++k) s += part[(size_t)k * len + i];
  out[(size_t)g * len + i] = s;
}

// Weight gradient: dW[o][ci][co] = sum_pos U[nbr[pos][o]][ci] * dY[pos][co], a contraction over tokens.  A workgroup
// takes one offset, one chunk of tokens and one CT x CT tile of the C x C matrix; 32-token tiles of the gathered U
// rows and of dY go through LDS row-major, both MFMA operands are transposing LDS reads of them.  Wave w owns the
// 16-row blocks w, w+4, .. of the tile.
template <int CT>
__global__ __launch_bounds__(256) void c_dw(const bf16_t *__restrict__ U, const bf16_t *__restrict__ dY,
                                            const int32_t *__restrict__ nbr, int N, int C, int chunk,
                                            float *__restrict__ part) {
  using G = TileGeom<CT>;
  __shared__ __align__(16) bf16_t su[G::ROW_ELEMS], sy[G::ROW_ELEMS];
  const int o = blockIdx.x, s = blockIdx.y, tiles = C / CT;
  const int ci0 = ((int)blockIdx.z / tiles) * CT, co0 = ((int)blockIdx.z % tiles) * CT;
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, quad = lane >> 4;
  constexpr int MB = CT / 16 / 4 > 0 ? CT / 16 / 4 : 1;  // 16-row blocks per wave
  constexpr int NBK = CT / 16;
  const bool wave_on = wid < CT / 16;
  f32x4 acc[MB][NBK];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int nb = 0; nb < NBK; ++nb) acc[a][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int b = s * chunk, e = min(N, b + chunk);
  for (int t0 = b; t0 < e; t0 += 32) {
    for (int it = threadIdx.x; it < G::ROW_ITEMS; it += 256) {
      const int row = it / (CT / 8), seg = it % (CT / 8);
      const int pos = t0 + row;
      const int src = pos < e ? nbr[(size_t)pos * 27 + o] : -1;
      const bf16x8 xu = src >= 0 ? ld8(U + (size_t)src * C + ci0 + 8 * seg) : zero8();
      const bf16x8 xy = (pos < e && src >= 0) ? ld8(dY + (size_t)pos * C + co0 + 8 * seg) : zero8();
      *reinterpret_cast<bf16x8 *>(su + G::row_off(row, seg)) = xu;
      *reinterpret_cast<bf16x8 *>(sy + G::row_off(row, seg)) = xy;
    }
    __syncthreads();
    if (wave_on) {
      bf16x8 av[MB];
#pragma unroll
      for (int a = 0; a < MB; ++a) av[a] = lds_tr_operand<CT>(su, wid + 4 * a);
#pragma unroll
      for (int nb = 0; nb < NBK; ++nb) {
        const bf16x8 bv = lds_tr_operand<CT>(sy, nb);
#pragma unroll
        for (int a = 0; a < MB; ++a) acc[a][nb] = mfma16(av[a], bv, acc[a][nb]);
      }
    }
    __syncthreads();
  }
  if (!wave_on) return;
  // C layout: lane holds column co = 16*nb + n, rows ci = 16*(wid + 4a) + 4*quad + i
  float *dst = part + ((size_t)s * 27 + o) * C * C;
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int nb = 0; nb < NBK; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        dst[(size_t)(ci0 + 16 * (wid + 4 * a) + 4 * quad + i) * C + co0 + 16 * nb + n] = acc[a][nb][i];
}

constexpr int PE_GROUPS = 32;  // first-level groups of the ordered dPE sum

struct ModPlan {
  size_t nbr, u, wt, y, dy, du, pw, ppe, ppe2, pb, total;
  int dw_chunks, dw_chunk, pe_chunks, pe_chunk;
};

ModPlan mod_plan(int N, int C, int m, bool backward) {
  ModPlan p{};
  size_t off = 0;
  auto take = [&](size_t n) { size_t r = off; off += align_up(n, 256); return r; };
  p.nbr = take((size_t)N * 27 * 4);
  p.u = take((size_t)N * C * 2);
  if (!backward) {
    p.wt = take((size_t)27 * C * C * 2);
    p.y = take((size_t)N * C * 4);
  } else {
    p.dy = take((size_t)N * C * 2);
    p.du = take((size_t)N * C * 4);
    p.dw_chunks = N > 0 ? (N + 2047) / 2048 : 1;
    if (p.dw_chunks > 32) p.dw_chunks = 32;
    p.dw_chunk = ((N + p.dw_chunks - 1) / p.dw_chunks + 31) / 32 * 32;
    if (p.dw_chunk < 32) p.dw_chunk = 32;
    p.pw = take((size_t)p.dw_chunks * 27 * C * C * 4);
    p.pe_chunks = N > 0 ? (N + 63) / 64 : 1;
    if (p.pe_chunks > 1024) p.pe_chunks = 1024;
    p.pe_chunk = (N + p.pe_chunks - 1) / p.pe_chunks;
    if (p.pe_chunk < 1) p.pe_chunk = 1;
    p.ppe = take((size_t)p.pe_chunks * m * m * m * C * 4);
    p.ppe2 = take((size_t)PE_GROUPS * m * m * m * C * 4);
    p.pb = take((size_t)DBIAS_PARTS * C * 4);
  }
  p.total = off;
  return p;
}

int check(const ssa_params_t *p, const ssa_blocks_t *b, int *C) {
  if (!p || !b) return SSA_ERR_NULL;
  if (p->n_tokens != b->N || p->n_batch != b->B || p->grid != b->G || p->m_cmp != b->m_cmp) return SSA_ERR_MISMATCH;
  if (p->n_heads_kv < 1 || p->head_dim < 1) return SSA_ERR_BAD_HEADS;
  if (p->dtype != SSA_BF16 || b->dims != 3) return SSA_ERR_UNSUPPORTED;  // the convolution is defined on the voxel grid
  const long long c = (long long)p->n_heads_kv * p->head_dim;
  if (c != 32 && c != 64 && c != 128 && c != 256) return SSA_ERR_UNSUPPORTED;
  if ((size_t)p->m_cmp * p->m_cmp * p->m_cmp * (size_t)c * 4 > 64 * 1024) return SSA_ERR_UNSUPPORTED;
  if ((long long)p->n_tokens * c >= (1ll << 31)) return SSA_ERR_BAD_SHAPE;
  *C = (int)c;
  return SSA_OK;
}

template <bool MIRROR>
void launch_conv(int C, const bf16_t *in, const int32_t *nbr, const bf16_t *Bw, const bf16_t *bias, int N, float *out,
                 hipStream_t s) {
  // 64 tokens per wavefront and up to 128 output channels per workgroup row (blockIdx.y picks the channel range)
  const dim3 grid((unsigned)((N + 255) / 256), (unsigned)(C > 128 ? C / 128 : 1));
  switch (C) {
    case 32: c_conv<32, MIRROR, 4, 2><<<grid, 256, 0, s>>>(in, nbr, Bw, bias, N, out); break;
    case 64: c_conv<64, MIRROR, 4, 4><<<grid, 256, 0, s>>>(in, nbr, Bw, bias, N, out); break;
    case 128: c_conv128<MIRROR, CONV_TOK><<<(unsigned)((N + CONV_TOK - 1) / CONV_TOK), 256, 0, s>>>(in, nbr, Bw, bias, N, out); break;
    default: c_conv<256, MIRROR, 4, 8><<<grid, 256, 0, s>>>(in, nbr, Bw, bias, N, out); break;
  }
}

}  // namespace

extern "C" size_t ssa_compress_workspace_bytes(const ssa_params_t *p, const ssa_blocks_t *b, int for_backward) {
  int C;
  if (check(p, b, &C) != SSA_OK) return 0;
  return mod_plan(b->N, C, b->m_cmp, for_backward != 0).total + 256;
}

extern "C" int ssa_compress_forward(const ssa_params_t *p, const ssa_blocks_t *b, const void *x,
                                    const ssa_cmp_weights_t *wts, void *x_cmp, void *ws_, size_t ws_bytes, void *stream) {
  int C;
  const int rc = check(p, b, &C);
  if (rc != SSA_OK) return rc;
  if (b->N == 0) return SSA_OK;
  if (!x || !wts || !wts->pe || !wts->w || !wts->bias || !x_cmp) return SSA_ERR_NULL;
  if (!aligned16(x, wts->pe, wts->w, wts->bias, x_cmp)) return SSA_ERR_ALIGNMENT;
  if (!ws_ || ws_bytes < ssa_compress_workspace_bytes(p, b, 0)) return SSA_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int N = b->N;
  const ModPlan pl = mod_plan(N, C, b->m_cmp, false);
  char *ws = (char *)align_up((size_t)ws_, 256);
  int32_t *nbr = (int32_t *)(ws + pl.nbr);
  bf16_t *U = (bf16_t *)(ws + pl.u), *Wt = (bf16_t *)(ws + pl.wt);
  float *Y = (float *)(ws + pl.y);
  ProfScope ps(PROF_CMP_MODULE, s);
  c_neighbors<<<(unsigned)(((size_t)N * 27 + 255) / 256), 256, 0, s>>>(b->sorted_keys, b->item_start, N, b->G, b->bits, nbr);
  const size_t items = (size_t)N * (C / 8);
  c_add_pe<<<(unsigned)((items + 255) / 256), 256, 0, s>>>((const bf16_t *)x, (const bf16_t *)wts->pe, b->perm, b->sorted_keys, N,
                                                             C, b->bits, b->m_cmp, U);
  c_transpose_w<<<(unsigned)(((size_t)27 * C * C + 255) / 256), 256, 0, s>>>((const bf16_t *)wts->w, C, Wt);
  launch_conv<false>(C, U, nbr, Wt, (const bf16_t *)wts->bias, N, Y, s);
  c_pool<<<b->Nc, 128, 0, s>>>(Y, b->cmp_start, C, (bf16_t *)x_cmp);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}

extern "C" int ssa_compress_backward(const ssa_params_t *p, const ssa_blocks_t *b, const void *x,
                                     const ssa_cmp_weights_t *wts, const float *dx_cmp, void *dx_accum, float *dpe,
                                     float *dw, float *dbias, void *ws_, size_t ws_bytes, void *stream) {
  int C;
  const int rc = check(p, b, &C);
  if (rc != SSA_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  if (b->N == 0) {  // no tokens: the parameter gradients are zero
    if (!dpe || !dw || !dbias) return SSA_ERR_NULL;
    const size_t plen0 = (size_t)b->m_cmp * b->m_cmp * b->m_cmp * C, wlen0 = (size_t)27 * C * C;
    c_sum_parts<<<(unsigned)((plen0 + 255) / 256), 256, 0, s>>>(nullptr, 0, 1, plen0, dpe);
    c_sum_parts<<<(unsigned)((wlen0 + 255) / 256), 256, 0, s>>>(nullptr, 0, 1, wlen0, dw);
    c_sum_parts<<<(C + 255) / 256, 256, 0, s>>>(nullptr, 0, 1, (size_t)C, dbias);
    return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
  }
  if (!x || !wts || !wts->pe || !wts->w || !wts->bias || !dx_cmp || !dx_accum || !dpe || !dw || !dbias) return SSA_ERR_NULL;
  if (!aligned16(x, wts->pe, wts->w, wts->bias, dx_cmp, dx_accum, dpe, dw, dbias)) return SSA_ERR_ALIGNMENT;
  if (!ws_ || ws_bytes < ssa_compress_workspace_bytes(p, b, 1)) return SSA_ERR_WORKSPACE;
  const int N = b->N, m = b->m_cmp;
  const ModPlan pl = mod_plan(N, C, m, true);
  char *ws = (char *)align_up((size_t)ws_, 256);
  int32_t *nbr = (int32_t *)(ws + pl.nbr);
  bf16_t *U = (bf16_t *)(ws + pl.u), *dY = (bf16_t *)(ws + pl.dy);
  float *dU = (float *)(ws + pl.du), *pw = (float *)(ws + pl.pw), *ppe = (float *)(ws + pl.ppe);
  float *ppe2 = (float *)(ws + pl.ppe2), *pb = (float *)(ws + pl.pb);
  ProfScope ps(PROF_CMP_MODULE_BWD, s);
  c_neighbors<<<(unsigned)(((size_t)N * 27 + 255) / 256), 256, 0, s>>>(b->sorted_keys, b->item_start, N, b->G, b->bits, nbr);
  const size_t items = (size_t)N * (C / 8);
  const unsigned igrid = (unsigned)((items + 255) / 256);
  c_add_pe<<<igrid, 256, 0, s>>>((const bf16_t *)x, (const bf16_t *)wts->pe, b->perm, b->sorted_keys, N, C, b->bits, m, U);
  c_expand<<<igrid, 256, 0, s>>>(dx_cmp, b->tok_cmp, b->cmp_start, N, C, dY);
  c_dbias_partial<<<dim3((C + 63) / 64, DBIAS_PARTS), 64, 0, s>>>(dx_cmp, b->Nc, C, pb);
  c_sum_parts<<<(C + 255) / 256, 256, 0, s>>>(pb, DBIAS_PARTS, 1, (size_t)C, dbias);
  // data gradient: dU[pos] = sum_o dY[token that took pos as neighbour o] * w[o]^T; w as given has c_out contiguous
  launch_conv<true>(C, dY, nbr, (const bf16_t *)wts->w, nullptr, N, dU, s);
  c_dx_accum<<<igrid, 256, 0, s>>>(dU, b->perm, N, C, (bf16_t *)dx_accum);
  const int rows = m * m * m;
  const size_t plen = (size_t)rows * C;
  c_dpe_partial<<<pl.pe_chunks, 128, plen * 4, s>>>(dU, b->sorted_keys, N, C, b->bits, m, pl.pe_chunk, ppe);
  c_sum_parts<<<dim3((unsigned)((plen + 255) / 256), PE_GROUPS), 256, 0, s>>>(ppe, pl.pe_chunks, PE_GROUPS, plen, ppe2);
  c_sum_parts<<<(unsigned)((plen + 255) / 256), 256, 0, s>>>(ppe2, PE_GROUPS, 1, plen, dpe);
  const int CT = C < 128 ? C : 128;
  const dim3 g(27, pl.dw_chunks, (C / CT) * (C / CT));
  switch (CT) {
    case 32: c_dw<32><<<g, 256, 0, s>>>(U, dY, nbr, N, C, pl.dw_chunk, pw); break;
    case 64: c_dw<64><<<g, 256, 0, s>>>(U, dY, nbr, N, C, pl.dw_chunk, pw); break;
    default: c_dw<128><<<g, 256, 0, s>>>(U, dY, nbr, N, C, pl.dw_chunk, pw); break;
  }
  const size_t wlen = (size_t)27 * C * C;
  c_sum_parts<<<(unsigned)((wlen + 255) / 256), 256, 0, s>>>(pw, pl.dw_chunks, 1, wlen, dw);
  return hipGetLastError() == hipSuccess ? SSA_OK : SSA_ERR_HIP;
}
