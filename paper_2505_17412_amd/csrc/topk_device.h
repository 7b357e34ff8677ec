// Wavefront-wide top-k over a score row held in LDS (paper: "The top-k selection blocks with the highest
// s_slc scores are selected").  Ties go to the lowest block id: each candidate is packed into one unsigned
// 64-bit key = (order-preserving image of the fp32 score) << 32 | (0xFFFFFFFF - index), so a plain unsigned
// maximum picks the largest score and, among equals, the smallest index.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ inline uint32_t ordered_bits(float f) {  // monotone map float -> uint32 (NaN excluded)
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, off);
    const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), off);
    const uint64_t o = ((uint64_t)hi << 32) | lo;
    v = o > v ? o : v;
  }
  return v;
}

// S[0..n): scores in LDS.  sel: LDS scratch of (n+31)/32 words.  Writes T ids (base + index) in ascending
// order, padded with -1.  Must be called by all 64 lanes of a one-wavefront workgroup region (uses
// __syncthreads only through the caller's convention: the workgroup is a single wavefront) -- or by one
// wavefront that owns S and sel exclusively when `single_wave_block` is false (then no barrier is used;
// LDS accesses of one wavefront are program-ordered).
__device__ inline void topk_wave(const float *S, int n, int T, int base, int32_t *out, uint32_t *sel) {
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
      const uint64_t key = ((uint64_t)ordered_bits(S[j]) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)j);
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
