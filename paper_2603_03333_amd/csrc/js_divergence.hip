// Distribution-level acceptance (Acceptance Criteria, "JS-Divergence-Based Criterion"): softmax of
// every path (Eq. (3)), the centroid = softmax of the mean of the K paths' logits (Eq. (5)), and the
// Jensen-Shannon divergences JS(p^(i) || pbar), JS(phat || pbar) that Eq. (6) compares.
//
// The contraction kernel has stored the scaled logits as lt[(pos * V + v) * K4 + i]; both passes here
// read that once, fully coalesced (see RowMap).  HBM-bound: 4 * K4 bytes per (position, vocabulary
// row) per pass, plus 4 bytes of the draft distribution in pass 2.
//
//   pass 1 (js_stats):  normalisers.  Z_i = max_i + ln sum_v exp(l_i[v] - max_i), with max_i already
//                       known from the argmax key of the row; for the mean logits lbar[v] the running
//                       (max, sum) pair, since their maximum is not known in advance.
//   pass 2 (js_terms):  with log p_i[v] = l_i[v] - Z_i, log pbar[v] = lbar[v] - Zbar and
//                       delta = log pbar - log p_i, the JS integrand is written without differences of
//                       nearly equal logarithms (js_term2).  The shorter log(p_i + pbar) - log p_i form
//                       was measured too: ten times the error (3e-7), so it is not used.
// Both passes are bound by the vector ALU, not by memory (a dozen plain instructions and three
// exp/log per stored logit): everything is kept in base 2 so that the hardware's exp2/log2 units are
// fed directly, whole chunks skip the bounds checks, and per-row work is dealt to the lanes of a group.
// Every reduction (lanes, wavefronts, chunks) runs in a fixed order: results are reproducible.
#include "kernels.hpp"

namespace dm {
namespace {

constexpr int JT = 1024;            // threads per workgroup (one workgroup = kJsChunk vocabulary rows of one position)

__device__ __forceinline__ float key_logit(unsigned long long key) {
  uint32_t u = (uint32_t)(key >> 32);
  u = (u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u;
  return __uint_as_float(u);
}

// All logarithms of the two passes are kept in base 2, the base of the hardware's exp and log units
// (v_exp_f32, v_log_f32: 1 ulp), so that no value is rescaled on its way in or out of them; the
// sums are turned into natural-log units once, at the end (factor ln 2).
constexpr float kLog2e = 1.44269504088896341f;
constexpr float kLn2 = 0.693147180559945309f;
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_hw(float x) { return __builtin_amdgcn_logf(x); }

// log2 of a sum kept in double, without the double-precision library routine (a few hundred instructions that every
// workgroup of pass 2 would run before its first load): the exponent is exact, and the hardware logarithm of the
// mantissa in [0.5, 1) is good to 6e-8 absolute, far below the rounding of the normaliser it goes into.
__device__ __forceinline__ double log2_of_sum(double s) {
  int e;
  const float f = frexpf((float)s, &e);
  return (double)e + (double)log2_hw(f);
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// One JS integrand in units of (ln 2) / 2, from log2 p, p, log2 q, q (q = centroid), written without
// differences of nearly equal logarithms: with delta = log2 q - log2 p and
//   a = log2(1 + 2^delta) = max(delta, 0) + log2(1 + 2^-|delta|)      (= 1 + log2(m / p), m = (p + q) / 2)
//   p log2(p/m) + q log2(q/m) = q delta - (p + q) (a - 1)
// (for p -> 0 it tends to q, for q -> 0 to p).
__device__ __forceinline__ float js_term2(float l2p, float p, float l2q, float q) {
  const float delta = l2q - l2p;
  const float a = fmaxf(delta, 0.f) + log2_hw(1.0f + exp2_hw(-fabsf(delta)));
  const float t = p + q;
  return fmaf(q, delta, fmaf(-t, a, t));
}

// Thread mapping of both passes.  A vocabulary row holds K4 floats; G = KP / 4 consecutive lanes
// (KP = K4 rounded up to a power of two) take 4 paths each of the same row, so one load instruction
// of a wavefront covers 64 / G consecutive rows = a contiguous piece of memory, and a lane keeps only
// 4 running sums.  The mean over the K paths of a row is a butterfly over the G lanes of its group.
// What is wanted once per row (the centroid's running normaliser in pass 1, the draft term in pass 2)
// would be computed by all G lanes of the group, since the lanes of a wavefront run in lockstep; rows
// are therefore taken in blocks of BL = min(G, 4) iterations and lane u of a group does that work for
// the block's u-th row.
template <int G>
struct RowMap {
  static constexpr int ROWS_PER_WAVE = 64 / G;
  static constexpr int ROWS_PER_ITER = (JT / 64) * ROWS_PER_WAVE;
  static constexpr int ITERS = kJsChunk / ROWS_PER_ITER;
  static constexpr int BL = G < 4 ? G : 4;
  static_assert(ITERS >= 1 && ITERS % BL == 0, "whole blocks of rows");
};

// Sum over the G consecutive lanes of a group (G = 1, 2, 4, 8, 16), result in every lane of the group,
// with data-parallel-primitive moves inside a row of 16 lanes (no LDS traffic): exchange with lane ^ 1,
// lane ^ 2, then the mirrored lane of the 8 (whose quad already holds its quad's sum), then of the 16.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
template <int G>
__device__ __forceinline__ float group_sum(float x) {
  if (G >= 2) x += dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]
  if (G >= 4) x += dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]
  if (G >= 8) x += dpp_move<0x141>(x);   // row_half_mirror
  if (G >= 16) x += dpp_move<0x140>(x);  // row_mirror
  return x;
}

// sum over the lanes that hold the same paths (same lane % G), result in every lane
template <int G>
__device__ __forceinline__ float column_sum(float x) {
#pragma unroll
  for (int off = G; off < 64; off <<= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// What both passes know about their place: the lane's four paths, its rows, which of them count.
template <int G, bool FULL>
struct LaneMap {
  int grp, i0;
  bool active;   // the lane's group of four paths exists in the store (i0 < K4)
  bool use[4];   // a head in use (not padding, whose slots are never written, nor the clean path); all true when FULL
  __device__ LaneMap(int lane, const JsGeom& g) {
    grp = lane % G;
    i0 = 4 * grp;
    active = i0 < g.K4;
#pragma unroll
    for (int j = 0; j < 4; ++j) use[j] = FULL || i0 + j < g.KU;
  }
};

// ---------------------------------------------------------------------------------------------- pass 1
// S_i += 2^(l2_i[v] - max2_i) for the lane's four paths and, for the rows dealt to this lane, the running
// (max, sum) of the mean logits.  CHECK: the chunk reaches past V (only the last chunk of a position).
template <int G, bool FULL, bool CHECK>
__device__ __forceinline__ void stats_loop(const float* __restrict__ base, int v_first, const JsGeom& g,
                                           const LaneMap<G, FULL>& lm, const float (&mx2)[4], float mean_scale,
                                           float (&S)[4], float& cmax, float& csum) {
  using RM = RowMap<G>;
  constexpr int BL = RM::BL;
  const float* row = base + (int64_t)v_first * g.K4;
  const int64_t step = (int64_t)RM::ROWS_PER_ITER * g.K4;
#pragma unroll 4 / BL
  for (int it0 = 0; it0 < RM::ITERS; it0 += BL) {
    float xbar2 = 0.f;
    bool mine = false;
#pragma unroll
    for (int u = 0; u < BL; ++u) {
      const int v = v_first + (it0 + u) * RM::ROWS_PER_ITER;
      const bool in = !CHECK || v < g.V;           // rows past the end re-read the last row with weight 0
      const float* src = CHECK ? base + (int64_t)(in ? v : g.V - 1) * g.K4 : row;
      row += step;
      const float4 qv = *reinterpret_cast<const float4*>(src);
      const float x[4] = {qv.x, qv.y, qv.z, qv.w};
      float xs = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {   // selects, not weights: an unused slot may hold anything, NaN included
        const float xj = lm.use[j] ? x[j] : 0.f;
        xs += xj;
        const float e = exp2_hw(fmaf(xj, kLog2e, -mx2[j]));
        S[j] += (lm.use[j] && in) ? e : 0.f;
      }
      xs = group_sum<G>(xs);
      if (lm.grp == u) {
        xbar2 = xs * mean_scale;
        mine = in;
      }
    }
    if (mine) {   // online (max, sum) of the mean logits over the rows of this lane
      const float m_new = fmaxf(cmax, xbar2);
      csum = fmaf(csum, exp2_hw(cmax - m_new), exp2_hw(xbar2 - m_new));
      cmax = m_new;
    }
  }
}

// FULL: the number of heads in use is 4 G, every lane's four paths exist (no per-path weights).
template <int G, bool FULL>
__global__ __launch_bounds__(JT) void js_stats_kernel(const float* __restrict__ lt,
                                                      const unsigned long long* __restrict__ keys,
                                                      float* __restrict__ part_a, JsGeom g, float scale) {
  using RM = RowMap<G>;
  constexpr int KP = 4 * G;
  __shared__ float red[JT / 64][KP + 2];
  const int pos = blockIdx.x, c = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = g.K, KU = g.KU;  // rows per position in the store / heads in use
  const LaneMap<G, FULL> lm(lane, g);

  float mx2[4], S[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    mx2[j] = lm.use[j] ? scale * key_logit(keys[(int64_t)pos * K + lm.i0 + j]) * kLog2e : 0.f;
    S[j] = 0.f;
  }
  // "Nothing yet" is a large negative finite number so that differences never become inf - inf.
  constexpr float kNone = -3.0e38f;
  float cmax = kNone, csum = 0.f;
  const float* base = lt + (int64_t)pos * g.V * g.K4 + (lm.active ? lm.i0 : 0);
  const int v_first = c * kJsChunk + wave * RM::ROWS_PER_WAVE + lane / G;
  const float mean_scale = kLog2e / (float)KU;   // mean over the heads, in base-2 units
  if ((c + 1) * kJsChunk <= g.V)
    stats_loop<G, FULL, false>(base, v_first, g, lm, mx2, mean_scale, S, cmax, csum);
  else
    stats_loop<G, FULL, true>(base, v_first, g, lm, mx2, mean_scale, S, cmax, csum);
  if (lm.grp >= RM::BL) {   // lanes that were dealt no rows
    cmax = kNone;
    csum = 0.f;
  }

  // wavefront level
  float wmax = cmax;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) wmax = fmaxf(wmax, __shfl_xor(wmax, off, 64));
  csum = csum * exp2_hw(cmax - wmax);
  csum = wave_sum(csum);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float t = column_sum<G>(S[j]);
    if (lane < G && lm.i0 + j < KU) red[wave][lm.i0 + j] = t;
  }
  if (lane == 0) {
    red[wave][KP] = wmax;
    red[wave][KP + 1] = csum;
  }
  __syncthreads();
  float* out = part_a + (int64_t)pos * g.KS * g.NC + c;  // record layout [pos][slot][chunk]
  if (tid < KU) {
    float t = red[0][tid];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) t += red[w][tid];
    out[(int64_t)tid * g.NC] = t;
  } else if (tid == 64) {
    float m = red[0][KP];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) m = fmaxf(m, red[w][KP]);
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < JT / 64; ++w) s += red[w][KP + 1] * exp2_hw(red[w][KP] - m);
    out[(int64_t)g.K4 * g.NC] = m;        // base-2 units: max over the chunk of log2(e) * mean logit
    out[(int64_t)(g.K4 + 1) * g.NC] = s;  // sum of 2^(that - max)
  }
}

// ---------------------------------------------------------------------------------------------- pass 2
template <int G, bool FULL, bool CHECK>
__device__ __forceinline__ void terms_loop(const float* __restrict__ base, const float* __restrict__ dp,
                                           int v_first, const JsGeom& g, const LaneMap<G, FULL>& lm,
                                           const float (&Z2)[4], float Zbar2, float mean_scale, bool draft_on,
                                           float (&J)[4], float& Jd) {
  using RM = RowMap<G>;
  constexpr int BL = RM::BL;
  const float* row = base + (int64_t)v_first * g.K4;
  const float* prow = dp + v_first;
  const int64_t step = (int64_t)RM::ROWS_PER_ITER * g.K4;
#pragma unroll 4 / BL
  for (int it0 = 0; it0 < RM::ITERS; it0 += BL) {
    float l2q_d = 0.f, q_d = 0.f, ph_d = 1.f;
    bool in_d = false;
#pragma unroll
    for (int u = 0; u < BL; ++u) {
      const int v = v_first + (it0 + u) * RM::ROWS_PER_ITER;
      const bool in = !CHECK || v < g.V;           // rows past the end re-read the last row with weight 0
      const int vc = in ? v : g.V - 1;
      const float4 qv = *reinterpret_cast<const float4*>(CHECK ? base + (int64_t)vc * g.K4 : row);
      const float ph = CHECK ? dp[vc] : *prow;
      row += step;
      prow += RM::ROWS_PER_ITER;
      const float x[4] = {qv.x, qv.y, qv.z, qv.w};
      float xs = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) xs += lm.use[j] ? x[j] : 0.f;   // selects: an unused slot may hold anything
      xs = group_sum<G>(xs);
      const float l2q = fmaf(xs, mean_scale, -Zbar2);
      const float q = exp2_hw(l2q);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float l2p = fmaf(lm.use[j] ? x[j] : 0.f, kLog2e, -Z2[j]);
        const float term = js_term2(l2p, exp2_hw(l2p), l2q, q);
        J[j] += (lm.use[j] && in) ? term : 0.f;
      }
      if (lm.grp == u) {
        l2q_d = l2q;
        q_d = q;
        ph_d = ph;
        in_d = in;
      }
    }
    // draft: log2 phat needs phat > 0; at phat = 0 the integrand is pbar (in units of ln2 / 2)
    const bool pos_ph = ph_d > 1e-37f;
    const float td = js_term2(log2_hw(pos_ph ? ph_d : 1.f), pos_ph ? ph_d : 0.f, l2q_d, q_d);
    Jd += (in_d && draft_on) ? (pos_ph ? td : q_d) : 0.f;
  }
}

template <int G, bool FULL>
__global__ __launch_bounds__(JT) void js_terms_kernel(const float* __restrict__ lt,
                                                      const unsigned long long* __restrict__ keys,
                                                      const float* __restrict__ part_a,
                                                      const float* __restrict__ draft_probs,
                                                      const int32_t* __restrict__ draft_ids,
                                                      float* __restrict__ part_b, JsGeom g, float scale) {
  using RM = RowMap<G>;
  constexpr int KP = 4 * G;
  __shared__ float Zs[KP + 1];
  __shared__ float red[JT / 64][KP + 1];
  const int pos = blockIdx.x, c = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = g.K, KU = g.KU;  // rows per position in the store / heads in use
  const LaneMap<G, FULL> lm(lane, g);

  // normalisers (base 2) from the partial sums of pass 1: 8 lanes per slot (a head, or the mean logits),
  // every lane adds every 8th chunk record (independent loads, all in flight together), then a butterfly
  // over the 8 lanes: a fixed order, the same in every workgroup
  const float* pa = part_a + (int64_t)pos * g.KS * g.NC;
  for (int slot = tid >> 3; slot <= KU; slot += JT / 8) {
    const int sub = tid & 7;
    if (slot < KU) {
      double s = 0.0;
      for (int cc = sub; cc < g.NC; cc += 8) s += (double)pa[(int64_t)slot * g.NC + cc];
#pragma unroll
      for (int off = 4; off >= 1; off >>= 1) s += __shfl_xor(s, off, 8);
      if (sub == 0) Zs[slot] = (float)((double)(scale * key_logit(keys[(int64_t)pos * K + slot]) * kLog2e) + log2_of_sum(s));
    } else {  // mean logits: chunk records are (max, sum of 2^(x - max))
      float m = -INFINITY;
      for (int cc = sub; cc < g.NC; cc += 8) m = fmaxf(m, pa[(int64_t)g.K4 * g.NC + cc]);
#pragma unroll
      for (int off = 4; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 8));
      // the rescaling factors in float (relative error 1e-7 per record, as good as the records themselves)
      double s = 0.0;
      for (int cc = sub; cc < g.NC; cc += 8)
        s += (double)(pa[(int64_t)(g.K4 + 1) * g.NC + cc] * exp2_hw(pa[(int64_t)g.K4 * g.NC + cc] - m));
#pragma unroll
      for (int off = 4; off >= 1; off >>= 1) s += __shfl_xor(s, off, 8);
      if (sub == 0) Zs[KP] = (float)((double)m + log2_of_sum(s));
    }
  }
  __syncthreads();
  float Z2[4], J[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    Z2[j] = lm.use[j] ? Zs[lm.i0 + j] : 0.f;
    J[j] = 0.f;
  }
  const float Zbar2 = Zs[KP];
  const bool draft_on = draft_ids[pos] >= 0 && lm.grp < RM::BL;
  float Jd = 0.f;
  const float* base = lt + (int64_t)pos * g.V * g.K4 + (lm.active ? lm.i0 : 0);
  const float* dp = draft_probs + (int64_t)pos * g.V;
  const int v_first = c * kJsChunk + wave * RM::ROWS_PER_WAVE + lane / G;
  const float mean_scale = kLog2e / (float)KU;
  if ((c + 1) * kJsChunk <= g.V)
    terms_loop<G, FULL, false>(base, dp, v_first, g, lm, Z2, Zbar2, mean_scale, draft_on, J, Jd);
  else
    terms_loop<G, FULL, true>(base, dp, v_first, g, lm, Z2, Zbar2, mean_scale, draft_on, J, Jd);

  constexpr float kUnit = 0.5f * kLn2;   // the sums are in units of (ln 2) / 2
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float t = column_sum<G>(J[j]);
    if (lane < G && lm.i0 + j < KU) red[wave][lm.i0 + j] = t;
  }
  Jd = wave_sum(Jd);
  if (lane == 0) red[wave][KP] = Jd;
  __syncthreads();
  float* out = part_b + (int64_t)pos * g.KS * g.NC + c;
  if (tid < KU) {
    float t = red[0][tid];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) t += red[w][tid];
    out[(int64_t)tid * g.NC] = t * kUnit;
  } else if (tid == 64) {
    float t = red[0][KP];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) t += red[w][KP];
    out[(int64_t)g.K4 * g.NC] = t * kUnit;
  }
}

}  // namespace

#define DM_JS_DISPATCH(KERNEL, ...)                                                          \
  do {                                                                                       \
    const dim3 grid((unsigned)g.P, (unsigned)g.NC), block(JT);                                \
    const int G = g.K4 <= 4 ? 1 : g.K4 <= 8 ? 2 : g.K4 <= 16 ? 4 : g.K4 <= 32 ? 8 : 16;       \
    const bool full = g.KU == 4 * G;                                                           \
    switch (G * 2 + (full ? 1 : 0)) {                                                         \
      case 2: KERNEL<1, false><<<grid, block, 0, stream>>>(__VA_ARGS__); break;               \
      case 3: KERNEL<1, true><<<grid, block, 0, stream>>>(__VA_ARGS__); break;                \
      case 4: KERNEL<2, false><<<grid, block, 0, stream>>>(__VA_ARGS__); break;               \
      case 5: KERNEL<2, true><<<grid, block, 0, stream>>>(__VA_ARGS__); break;                \
      case 8: KERNEL<4, false><<<grid, block, 0, stream>>>(__VA_ARGS__); break;               \
      case 9: KERNEL<4, true><<<grid, block, 0, stream>>>(__VA_ARGS__); break;                \
      case 16: KERNEL<8, false><<<grid, block, 0, stream>>>(__VA_ARGS__); break;              \
      case 17: KERNEL<8, true><<<grid, block, 0, stream>>>(__VA_ARGS__); break;               \
      case 32: KERNEL<16, false><<<grid, block, 0, stream>>>(__VA_ARGS__); break;             \
      default: KERNEL<16, true><<<grid, block, 0, stream>>>(__VA_ARGS__); break;              \
    }                                                                                         \
  } while (0)

hipError_t launch_js_stats(const float* lt, const unsigned long long* keys, float* part_a, const JsGeom& g,
                           float scale, hipStream_t stream) {
  if (g.K < 1 || g.K > kJsMaxK || g.KU < 1 || g.KU > g.K || g.P < 1 || g.NC < 1 || g.NC > 65535) return hipErrorInvalidValue;
  DM_JS_DISPATCH(js_stats_kernel, lt, keys, part_a, g, scale);
  return hipGetLastError();
}

hipError_t launch_js_terms(const float* lt, const unsigned long long* keys, const float* part_a,
                           const float* draft_probs, const int32_t* draft_ids, float* part_b, const JsGeom& g,
                           float scale, hipStream_t stream) {
  if (g.K < 1 || g.K > kJsMaxK || g.KU < 1 || g.KU > g.K || g.P < 1 || g.NC < 1 || g.NC > 65535) return hipErrorInvalidValue;
  DM_JS_DISPATCH(js_terms_kernel, lt, keys, part_a, draft_probs, draft_ids, part_b, g, scale);
  return hipGetLastError();
}

}  // namespace dm
