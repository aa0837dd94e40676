// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) as the random source of the keep-masks
// of Eq. (1).  Counter (j >> 2, row, path, step), key = 64-bit sequence seed; dimension j
// takes output word (j & 3); keep iff word >= floor(p * 2^32).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dm {

struct Philox4 {
  uint32_t w[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32 x 32 -> 64 bit multiply per product (v_mad_u64_u32) instead of a high and a low multiply
    const uint64_t p0 = (uint64_t)M0 * c0, p1 = (uint64_t)M1 * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0;
    c1 = lo1;
    c2 = n2;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  Philox4 o;
  o.w[0] = c0;
  o.w[1] = c1;
  o.w[2] = c2;
  o.w[3] = c3;
  return o;
}

// 8 keep bits for dimensions 8*o .. 8*o+7 of (row word t, path i): bit e = keep(8*o + e).
__device__ __forceinline__ uint32_t keep_bits8(uint32_t o, uint32_t t, uint32_t i, uint32_t step,
                                               uint32_t k0, uint32_t k1, uint32_t thr) {
  const Philox4 a = philox4x32_10(2u * o, t, i, step, k0, k1);
  const Philox4 b = philox4x32_10(2u * o + 1u, t, i, step, k0, k1);
  uint32_t bits = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    bits |= (a.w[e] >= thr ? 1u : 0u) << e;
    bits |= (b.w[e] >= thr ? 1u : 0u) << (4 + e);
  }
  return bits;
}

// ---- sampled path tokens: Gumbel-max draw from Softmax(l / tau) ------------------------------
// The paper remarks that a path's token may be selected by sampling instead of the arg max.
// y = argmax_v (l[v] / tau + g[v]) with g = -ln(-ln u) is a draw from Softmax(l / tau); u[v] comes
// from a Philox stream of its own: counter (v >> 2, row, path, step), key = sequence seed +
// 0x9E3779B97F4A7C15 (mod 2^64), word v & 3, u = ((w >> 9) + 1/2) 2^-23 (exact in float, never 0 or 1).
constexpr uint64_t kSampleKeyOffset = 0x9E3779B97F4A7C15ull;

// g = -ln(-ln u).  The largest g come from u next to 1, where -ln u has to be accurate relative to
// its own size: there it is the series of -ln(1 - c) in c = 1 - u (exact in float); elsewhere the
// hardware logarithm (base 2, 1 ulp) is enough.
__device__ __forceinline__ float gumbel_from_word(uint32_t w) {
  const float k = (float)(w >> 9);
  const float u = (k + 0.5f) * 1.1920928955078125e-07f;             // 2^-23
  const float c = (8388607.5f - k) * 1.1920928955078125e-07f;       // 1 - u, exact
  const float series = c * (1.0f + c * (0.5f + c * (0.333333343f + c * 0.25f)));
  const float direct = -0.693147180559945309f * __builtin_amdgcn_logf(u);
  const float e = (c <= 0.015625f) ? series : direct;               // -ln u
  return -0.693147180559945309f * __builtin_amdgcn_logf(e);
}

// Which stream a masked row draws from.
struct RowRng {
  uint32_t k0, k1, t, i;
  bool on;   // false: padding row, or the clean last path (plain arg max)
};

}  // namespace dm
