// Distribution-level acceptance (Acceptance Criteria, "JS-Divergence-Based Criterion"): softmax of
// every path (Eq. (3)), the centroid = softmax of the mean of the K paths' logits (Eq. (5)), and the
// Jensen-Shannon divergences JS(p^(i) || pbar), JS(phat || pbar) that Eq. (6) compares.
//
// The contraction kernel has stored the scaled logits as lt[(pos * V + v) * K4 + i]; both passes here
// read that once, coalesced (a thread takes one vocabulary row v = K4 contiguous floats, consecutive
// threads take consecutive rows).  HBM-bound: 4 * K4 bytes per (position, vocabulary row) per pass.
//
//   pass 1 (js_stats):  normalisers.  Z_i = max_i + ln sum_v exp(l_i[v] - max_i), with max_i already
//                       known from the argmax key of the row; for the mean logits lbar[v] the running
//                       (max, sum) pair, since their maximum is not known in advance.
//   pass 2 (js_terms):  with ln p_i[v] = l_i[v] - Z_i, ln pbar[v] = lbar[v] - Zbar and
//                       delta = ln pbar - ln p_i, the JS integrand is written without differences of
//                       nearly equal logarithms:
//                         a = ln((1 + e^delta) / 2) = ln(m / p_i),   m = (p_i + pbar) / 2
//                         p_i ln(p_i/m)/2 + pbar ln(pbar/m)/2 = (pbar * delta - (p_i + pbar) * a) / 2
//                       (for p_i -> 0 it tends to pbar ln2 / 2, for pbar -> 0 to p_i ln2 / 2).
// Every reduction (lanes, wavefronts, chunks) runs in a fixed order: results are reproducible.
#include "kernels.hpp"

namespace dm {
namespace {

constexpr int JT = 256;             // threads per workgroup
constexpr int JV = kJsChunk / JT;   // vocabulary rows per thread

__device__ __forceinline__ float key_logit(unsigned long long key) {
  uint32_t u = (uint32_t)(key >> 32);
  u = (u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u;
  return __uint_as_float(u);
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// ln((1 + e^x) / 2) without overflow
__device__ __forceinline__ float log_half_1pexp(float x) {
  return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x))) - 0.693147180559945309f;
}

// one JS integrand from ln p, ln q (q = centroid) and the probabilities themselves
__device__ __forceinline__ float js_term(float lp, float p, float lq, float q) {
  const float delta = lq - lp;
  const float a = log_half_1pexp(delta);
  return 0.5f * (q * delta - (p + q) * a);
}

template <int KP>
__device__ __forceinline__ void load_row(const float* __restrict__ src, int K4, float (&x)[KP]) {
#pragma unroll
  for (int g = 0; g < KP / 4; ++g) {
    if (4 * g < K4) {
      const float4 q = *reinterpret_cast<const float4*>(src + 4 * g);
      x[4 * g + 0] = q.x;
      x[4 * g + 1] = q.y;
      x[4 * g + 2] = q.z;
      x[4 * g + 3] = q.w;
    }
  }
}

template <int KP>
__global__ __launch_bounds__(JT) void js_stats_kernel(const float* __restrict__ lt,
                                                      const unsigned long long* __restrict__ keys,
                                                      float* __restrict__ part_a, JsGeom g, float scale) {
  __shared__ float red[JT / 64][KP + 2];
  const int pos = blockIdx.x, c = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = g.K;

  float mx[KP], S[KP];
#pragma unroll
  for (int i = 0; i < KP; ++i) {
    mx[i] = (i < K) ? scale * key_logit(keys[(int64_t)pos * K + i]) : 0.f;
    S[i] = 0.f;
  }
  float cb[JV];
  float cmax = -INFINITY;
  const float* base = lt + (int64_t)pos * g.V * g.K4;
#pragma unroll
  for (int j = 0; j < JV; ++j) {
    const int v = c * kJsChunk + j * JT + tid;
    cb[j] = -INFINITY;
    if (v < g.V) {
      float x[KP];
      load_row<KP>(base + (int64_t)v * g.K4, g.K4, x);
      float xs = 0.f;
#pragma unroll
      for (int i = 0; i < KP; ++i)
        if (i < K) {
          xs += x[i];
          S[i] += expf(x[i] - mx[i]);
        }
      cb[j] = xs / (float)K;
      cmax = fmaxf(cmax, cb[j]);
    }
  }
  float csum = 0.f;
#pragma unroll
  for (int j = 0; j < JV; ++j)
    if (cb[j] != -INFINITY) csum += expf(cb[j] - cmax);

  // wavefront level
  float wmax = cmax;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) wmax = fmaxf(wmax, __shfl_xor(wmax, off, 64));
  csum = (cmax == -INFINITY) ? 0.f : csum * expf(cmax - wmax);
  csum = wave_sum(csum);
#pragma unroll
  for (int i = 0; i < KP; ++i)
    if (i < K) {
      const float t = wave_sum(S[i]);
      if (lane == 0) red[wave][i] = t;
    }
  if (lane == 0) {
    red[wave][KP] = wmax;
    red[wave][KP + 1] = csum;
  }
  __syncthreads();
  float* out = part_a + ((int64_t)pos * g.NC + c) * g.KS;
  if (tid < K) {
    float t = red[0][tid];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) t += red[w][tid];
    out[tid] = t;
  } else if (tid == 64) {
    float m = red[0][KP];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) m = fmaxf(m, red[w][KP]);
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < JT / 64; ++w)
      if (red[w][KP] != -INFINITY) s += red[w][KP + 1] * expf(red[w][KP] - m);
    out[g.K4] = m;
    out[g.K4 + 1] = s;
  }
}

template <int KP>
__global__ __launch_bounds__(JT) void js_terms_kernel(const float* __restrict__ lt,
                                                      const unsigned long long* __restrict__ keys,
                                                      const float* __restrict__ part_a,
                                                      const float* __restrict__ draft_probs,
                                                      const int32_t* __restrict__ draft_ids,
                                                      float* __restrict__ part_b, JsGeom g, float scale) {
  __shared__ float Zs[KP + 1];
  __shared__ float red[JT / 64][KP + 1];
  const int pos = blockIdx.x, c = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = g.K;

  // normalisers from the partial sums of pass 1, chunks in ascending order
  const float* pa = part_a + (int64_t)pos * g.NC * g.KS;
  if (tid < K) {
    double s = 0.0;
    for (int cc = 0; cc < g.NC; ++cc) s += (double)pa[cc * g.KS + tid];
    Zs[tid] = (float)((double)(scale * key_logit(keys[(int64_t)pos * K + tid])) + log(s));
  } else if (tid == 64) {
    float m = -INFINITY;
    for (int cc = 0; cc < g.NC; ++cc) m = fmaxf(m, pa[cc * g.KS + g.K4]);
    double s = 0.0;
    for (int cc = 0; cc < g.NC; ++cc) s += (double)pa[cc * g.KS + g.K4 + 1] * exp((double)pa[cc * g.KS + g.K4] - (double)m);
    Zs[KP] = (float)((double)m + log(s));
  }
  __syncthreads();
  float Z[KP], J[KP];
#pragma unroll
  for (int i = 0; i < KP; ++i) {
    Z[i] = (i < K) ? Zs[i] : 0.f;
    J[i] = 0.f;
  }
  const float Zbar = Zs[KP];
  const bool has_draft = draft_ids[pos] >= 0;
  float Jd = 0.f;
  const float* base = lt + (int64_t)pos * g.V * g.K4;
  const float* dp = draft_probs + (int64_t)pos * g.V;
#pragma unroll 2
  for (int j = 0; j < JV; ++j) {
    const int v = c * kJsChunk + j * JT + tid;
    if (v < g.V) {
      float x[KP];
      load_row<KP>(base + (int64_t)v * g.K4, g.K4, x);
      float xs = 0.f;
#pragma unroll
      for (int i = 0; i < KP; ++i)
        if (i < K) xs += x[i];
      const float lq = xs / (float)K - Zbar;
      const float q = expf(lq);
#pragma unroll
      for (int i = 0; i < KP; ++i)
        if (i < K) {
          const float lp = x[i] - Z[i];
          J[i] += js_term(lp, expf(lp), lq, q);
        }
      if (has_draft) {
        const float ph = dp[v];
        Jd += (ph > 0.f) ? js_term(logf(ph), ph, lq, q) : 0.5f * 0.693147180559945309f * q;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < KP; ++i)
    if (i < K) {
      const float t = wave_sum(J[i]);
      if (lane == 0) red[wave][i] = t;
    }
  Jd = wave_sum(Jd);
  if (lane == 0) red[wave][KP] = Jd;
  __syncthreads();
  float* out = part_b + ((int64_t)pos * g.NC + c) * g.KS;
  if (tid < K) {
    float t = red[0][tid];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) t += red[w][tid];
    out[tid] = t;
  } else if (tid == 64) {
    float t = red[0][KP];
#pragma unroll
    for (int w = 1; w < JT / 64; ++w) t += red[w][KP];
    out[g.K4] = t;
  }
}

}  // namespace

#define DM_JS_DISPATCH(KERNEL, ...)                                                        \
  do {                                                                                     \
    const dim3 grid((unsigned)g.P, (unsigned)g.NC), block(JT);                              \
    if (g.K4 <= 4) KERNEL<4><<<grid, block, 0, stream>>>(__VA_ARGS__);                      \
    else if (g.K4 <= 8) KERNEL<8><<<grid, block, 0, stream>>>(__VA_ARGS__);                 \
    else if (g.K4 <= 16) KERNEL<16><<<grid, block, 0, stream>>>(__VA_ARGS__);               \
    else if (g.K4 <= 32) KERNEL<32><<<grid, block, 0, stream>>>(__VA_ARGS__);               \
    else KERNEL<64><<<grid, block, 0, stream>>>(__VA_ARGS__);                               \
  } while (0)

hipError_t launch_js_stats(const float* lt, const unsigned long long* keys, float* part_a, const JsGeom& g,
                           float scale, hipStream_t stream) {
  if (g.K < 1 || g.K > kJsMaxK || g.P < 1 || g.NC < 1 || g.NC > 65535) return hipErrorInvalidValue;
  DM_JS_DISPATCH(js_stats_kernel, lt, keys, part_a, g, scale);
  return hipGetLastError();
}

hipError_t launch_js_terms(const float* lt, const unsigned long long* keys, const float* part_a,
                           const float* draft_probs, const int32_t* draft_ids, float* part_b, const JsGeom& g,
                           float scale, hipStream_t stream) {
  if (g.K < 1 || g.K > kJsMaxK || g.P < 1 || g.NC < 1 || g.NC > 65535) return hipErrorInvalidValue;
  DM_JS_DISPATCH(js_terms_kernel, lt, keys, part_a, draft_probs, draft_ids, part_b, g, scale);
  return hipGetLastError();
}

}  // namespace dm
