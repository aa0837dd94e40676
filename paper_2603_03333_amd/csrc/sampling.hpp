// Helpers of the sampling epilogues of the contraction kernels (see philox.hpp for the construction).
#pragma once
#include "kernels.hpp"
#include "philox.hpp"

namespace dm {

// Stream of masked row m (row index = (b*T + t)*K + i); off for padding rows and for a clean last path.
__device__ __forceinline__ RowRng make_row_rng(const SampleCfg& sc, int64_t m, int64_t M) {
  RowRng r{0u, 0u, 0u, 0u, false};
  if (sc.seeds == nullptr || m >= M) return r;
  const int TK = sc.T * sc.K;
  int64_t b;
  int rem;
  if (M <= 0x7fffffff) {  // every practical size: 32-bit divisions (the 64-bit one is ~100 instructions)
    const uint32_t b32 = (uint32_t)m / (uint32_t)TK;
    b = b32;
    rem = (int)((uint32_t)m - b32 * (uint32_t)TK);
  } else {
    b = m / TK;
    rem = (int)(m - b * TK);
  }
  const int t = rem / sc.K;
  const int i = rem - t * sc.K;
  const uint64_t key = sc.seeds[b] + kSampleKeyOffset;
  r.k0 = (uint32_t)key;
  r.k1 = (uint32_t)(key >> 32);
  r.t = (uint32_t)t;
  r.i = (uint32_t)i;
  r.on = !(sc.clean_last && i == sc.K - 1);
  return r;
}

// Whether masked row m draws its token (false: padding row, or the clean last path).
__device__ __forceinline__ bool row_draws(const SampleCfg& sc, int64_t m, int64_t M) {
  if (sc.seeds == nullptr || m >= M) return false;
  if (!sc.clean_last) return true;
  const int i = M <= 0x7fffffff ? (int)((uint32_t)m % (uint32_t)sc.K) : (int)(m % sc.K);
  return i != sc.K - 1;
}

// Gumbel noise of vocabulary entries v4 .. v4+3 (v4 a multiple of 4) for one row: one Philox call.
__device__ __forceinline__ void gumbel4(const RowRng& r, uint32_t v4, uint32_t step, float (&g)[4]) {
  const Philox4 x = philox4x32_10(v4 >> 2, r.t, r.i, step, r.k0, r.k1);
#pragma unroll
  for (int e = 0; e < 4; ++e) g[e] = gumbel_from_word(x.w[e]);
}

}  // namespace dm
