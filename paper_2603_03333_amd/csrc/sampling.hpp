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
  const int64_t b = m / TK;
  const int rem = (int)(m - b * TK);
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

// Gumbel noise of vocabulary entries v4 .. v4+3 (v4 a multiple of 4) for one row: one Philox call.
__device__ __forceinline__ void gumbel4(const RowRng& r, uint32_t v4, uint32_t step, float (&g)[4]) {
  const Philox4 x = philox4x32_10(v4 >> 2, r.t, r.i, step, r.k0, r.k1);
#pragma unroll
  for (int e = 0; e < 4; ++e) g[e] = gumbel_from_word(x.w[e]);
}

}  // namespace dm
