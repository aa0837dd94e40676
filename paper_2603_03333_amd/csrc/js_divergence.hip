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
//   pass 2 (js_terms):  with ln p_i[v] = l_i[v] - Z_i, ln pbar[v] = lbar[v] - Zbar and
//                       delta = ln pbar - ln p_i, the JS integrand is written without differences of
//                       nearly equal logarithms:
//                         a = ln((1 + e^delta) / 2) = ln(m / p_i),   m = (p_i + pbar) / 2
//                         p_i ln(p_i/m)/2 + pbar ln(pbar/m)/2 = (pbar * delta - (p_i + pbar) * a) / 2
//                       (for p_i -> 0 it tends to pbar ln2 / 2, for pbar -> 0 to p_i ln2 / 2).  The
//                       shorter a = ln(p_i + pbar) - ln 2 - ln p_i was measured too: 3 % faster, ten
//                       times the error (3e-7), so it is not used.
// Every reduction (lanes, wavefronts, chunks) runs in a fixed order: results are reproducible.
#include "kernels.hpp"

namespace dm {
namespace {

constexpr int JT = 256;             // threads per workgroup

__device__ __forceinline__ float key_logit(unsigned long long key) {
  uint32_t u = (uint32_t)(key >> 32);
  u = (u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u;
  return __uint_as_float(u);
}

// e^x and ln x on the hardware's base-2 units (1 ulp each; the argument scaling adds a relative
// error of about |x| * 1e-7 to e^x, far inside what Eq. (6) needs).  ln is used on [1, 2] and on
// probabilities above the smallest normal float.
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }
__device__ __forceinline__ float fast_log(float x) { return __builtin_amdgcn_logf(x) * 0.693147180559945309f; }

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// ln((1 + e^x) / 2) without overflow
__device__ __forceinline__ float log_half_1pexp(float x) {
  return fmaxf(x, 0.f) + fast_log(1.0f + fast_exp(-fabsf(x))) - 0.693147180559945309f;
}

// one JS integrand from ln p, ln q (q = centroid) and the probabilities themselves
__device__ __forceinline__ float js_term(float lp, float p, float lq, float q) {
  const float delta = lq - lp;
  const float a = log_half_1pexp(delta);
  return 0.5f * (q * delta - (p + q) * a);
}

// Thread mapping of both passes.  A vocabulary row holds K4 floats; G = KP / 4 consecutive lanes
// (KP = K4 rounded up to a power of two) take 4 paths each of the same row, so one load instruction
// of a wavefront covers 64 / G consecutive rows = a contiguous piece of memory, and a lane keeps only
// 4 running sums.  The mean over the K paths of a row is a butterfly over the G lanes of its group;
// lane 0 of the group then owns the row's centroid and draft terms.
template <int G>
struct RowMap {
  static constexpr int ROWS_PER_WAVE = 64 / G;
  static constexpr int ROWS_PER_ITER = (JT / 64) * ROWS_PER_WAVE;
  static constexpr int ITERS = kJsChunk / ROWS_PER_ITER;
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

// FULL: the number of heads in use is 4 G, every lane's four paths exist (no per-path predicates).
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
  const int grp = lane % G, rl = lane / G;
  const int i0 = 4 * grp;             // first path of this lane
  const bool active = i0 < g.K4;

  float mx[4], S[4];
  bool use[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    use[j] = FULL || i0 + j < KU;
    mx[j] = use[j] ? scale * key_logit(keys[(int64_t)pos * K + i0 + j]) : 0.f;
    S[j] = 0.f;
  }
  // centroid: running (max, sum of exp relative to it); kept by every lane of a group, lane 0's is used.
  // "Nothing yet" is a large negative finite number so that differences never become inf - inf.
  constexpr float kNone = -3.0e38f;
  float cmax = kNone, csum = 0.f;
  const float* base = lt + (int64_t)pos * g.V * g.K4 + (active ? i0 : 0);
  const int v_first = c * kJsChunk + wave * RM::ROWS_PER_WAVE + rl;
  const float inv_k = 1.0f / (float)KU;
  const bool exact_inv = (KU & (KU - 1)) == 0;  // then x * (1/K) is the correctly rounded x / K
#pragma unroll 4
  for (int it = 0; it < RM::ITERS; ++it) {
    const int v = v_first + it * RM::ROWS_PER_ITER;
    const bool in = v < g.V;                       // only the last chunk has rows past the end:
    const int vc = in ? v : g.V - 1;               // they re-read the last row with weight 0
    const float4 q = *reinterpret_cast<const float4*>(base + (int64_t)vc * g.K4);
    const float x[4] = {q.x, q.y, q.z, q.w};
    const float wgt = (in && active) ? 1.f : 0.f;
    float xs = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float xj = (use[j] && active) ? x[j] : 0.f;
      xs += xj;
      S[j] += (use[j] ? wgt : 0.f) * fast_exp(xj - mx[j]);
    }
    xs = group_sum<G>(xs);
    const float xbar = in ? (exact_inv ? xs * inv_k : xs / (float)KU) : kNone;
    const float m_new = fmaxf(cmax, xbar);
    csum = csum * fast_exp(cmax - m_new) + (in ? 1.f : 0.f) * fast_exp(xbar - m_new);
    cmax = m_new;
  }
  if (grp != 0) {
    cmax = kNone;
    csum = 0.f;
  }

  // wavefront level
  float wmax = cmax;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) wmax = fmaxf(wmax, __shfl_xor(wmax, off, 64));
  csum = csum * fast_exp(cmax - wmax);
  csum = wave_sum(csum);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float t = column_sum<G>(S[j]);
    if (lane < G && i0 + j < KU) red[wave][i0 + j] = t;
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
    for (int w = 0; w < JT / 64; ++w) s += red[w][KP + 1] * fast_exp(red[w][KP] - m);
    out[(int64_t)g.K4 * g.NC] = m;
    out[(int64_t)(g.K4 + 1) * g.NC] = s;
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
  const int grp = lane % G, rl = lane / G;
  const int i0 = 4 * grp;
  const bool active = i0 < g.K4;

  // normalisers from the partial sums of pass 1: 8 lanes per slot (a head, or the mean logits), every
  // lane adds every 8th chunk record (independent loads, all in flight together), then a butterfly over
  // the 8 lanes: a fixed order, the same in every workgroup
  const float* pa = part_a + (int64_t)pos * g.KS * g.NC;
  for (int slot = tid >> 3; slot <= KU; slot += JT / 8) {
    const int sub = tid & 7;
    if (slot < KU) {
      double s = 0.0;
      for (int cc = sub; cc < g.NC; cc += 8) s += (double)pa[(int64_t)slot * g.NC + cc];
#pragma unroll
      for (int off = 4; off >= 1; off >>= 1) s += __shfl_xor(s, off, 8);
      if (sub == 0) Zs[slot] = (float)((double)(scale * key_logit(keys[(int64_t)pos * K + slot])) + log(s));
    } else {  // mean logits: chunk records are (max, sum of exp relative to that max)
      float m = -INFINITY;
      for (int cc = sub; cc < g.NC; cc += 8) m = fmaxf(m, pa[(int64_t)g.K4 * g.NC + cc]);
#pragma unroll
      for (int off = 4; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 8));
      double s = 0.0;
      for (int cc = sub; cc < g.NC; cc += 8)
        s += (double)pa[(int64_t)(g.K4 + 1) * g.NC + cc] * exp((double)pa[(int64_t)g.K4 * g.NC + cc] - (double)m);
#pragma unroll
      for (int off = 4; off >= 1; off >>= 1) s += __shfl_xor(s, off, 8);
      if (sub == 0) Zs[KP] = (float)((double)m + log(s));
    }
  }
  __syncthreads();
  float Z[4], J[4];
  bool use[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    use[j] = FULL || i0 + j < KU;
    Z[j] = use[j] ? Zs[i0 + j] : 0.f;
    J[j] = 0.f;
  }
  const float Zbar = Zs[KP];
  const bool draft_on = draft_ids[pos] >= 0 && grp == 0;
  float Jd = 0.f;
  const float* base = lt + (int64_t)pos * g.V * g.K4 + (active ? i0 : 0);
  const float* dp = draft_probs + (int64_t)pos * g.V;
  const int v_first = c * kJsChunk + wave * RM::ROWS_PER_WAVE + rl;
  const float inv_k = 1.0f / (float)KU;
  const bool exact_inv = (KU & (KU - 1)) == 0;
#pragma unroll 4
  for (int it = 0; it < RM::ITERS; ++it) {
    const int v = v_first + it * RM::ROWS_PER_ITER;
    const bool in = v < g.V;                       // rows past the end re-read the last row with weight 0
    const int vc = in ? v : g.V - 1;
    const float4 qv = *reinterpret_cast<const float4*>(base + (int64_t)vc * g.K4);
    const float ph = dp[vc];
    const float x[4] = {qv.x, qv.y, qv.z, qv.w};
    const float wgt = (in && active) ? 1.f : 0.f;
    float xs = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) xs += (use[j] && active) ? x[j] : 0.f;
    xs = group_sum<G>(xs);
    const float lq = (exact_inv ? xs * inv_k : xs / (float)KU) - Zbar;
    const float q = fast_exp(lq);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float lp = ((use[j] && active) ? x[j] : 0.f) - Z[j];
      J[j] += (use[j] ? wgt : 0.f) * js_term(lp, fast_exp(lp), lq, q);
    }
    // draft: ln phat needs phat > 0; at phat = 0 the integrand is pbar ln2 / 2
    const bool pos_ph = ph > 1e-37f;
    const float td = js_term(fast_log(pos_ph ? ph : 1.f), pos_ph ? ph : 0.f, lq, q);
    Jd += (in && draft_on) ? (pos_ph ? td : 0.5f * 0.693147180559945309f * q) : 0.f;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float t = column_sum<G>(J[j]);
    if (lane < G && i0 + j < KU) red[wave][i0 + j] = t;
  }
  Jd = wave_sum(Jd);
  if (lane == 0) red[wave][KP] = Jd;
  __syncthreads();
  float* out = part_b + (int64_t)pos * g.KS * g.NC + c;
  if (tid < KU) {
    float t = red[0][tid];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) t += red[w][tid];
    out[(int64_t)tid * g.NC] = t;
  } else if (tid == 64) {
    float t = red[0][KP];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) t += red[w][KP];
    out[(int64_t)g.K4 * g.NC] = t;
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
