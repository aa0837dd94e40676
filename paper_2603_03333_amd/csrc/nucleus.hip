// Sampled path tokens restricted to the nucleus (top-p set) of Softmax(l / tau) - the paper names
// nucleus sampling (Holtzman et al.) as the alternative to the arg max for a path's token.
//
// For one masked row with logits l[v] (stored by the contraction kernel) and maximum lmax, let
// t[v] = (lmax - l[v]) / tau >= 0, so that the row's probabilities are proportional to e^-t.
// The nucleus is { v : t[v] <= t* }, t* being the smallest value for which the tokens with
// t <= t* carry at least top_p of the row's mass (tokens exactly as probable as the last one
// needed are all in).  Masses are summed as 64-bit integers, floor(e^-t * 2^44): integer sums
// do not depend on the order of the additions, so every run makes the same decisions.
//
// t* is found by a radix search over t in fixed point, 24 bits in units of 2^-19 (order_key: the
// whole range in which a token has any mass; at temperatures up to 1 a finer resolution than the
// float32 logits are good for; tokens that share a key count as equally probable), 8 bits per level:
//   nucleus_hist_kernel   per (position, chunk of vocabulary rows): the mass of every 8-bit digit
//                         among the row's elements that match the digits fixed so far - first in
//                         LDS (one histogram per path of the position), then the non-empty bins
//                         are added to the row's 256 bins in memory;
//   nucleus_scan_kernel   per row: walk the bins in order of growing t until the target mass is
//                         reached; that digit is fixed, the mass below it carried on, the bins
//                         cleared for the next level.  Level 0 also turns top_p into the target.
// After three levels the key of t* is known.
//   nucleus_draw_kernel   arg max of l[v] / tau + Gumbel noise over the nucleus (the same noise
//                         stream as the unrestricted draw, so top_p -> 1 gives that draw), merged
//                         into a second array of packed keys that the acceptance step then reads.
// All three are bound by reading the logit store: 4 * K4 bytes per (position, vocabulary row) per pass.
#include "kernels.hpp"
#include "sampling.hpp"

namespace dm {
namespace {

constexpr int NT = 256;          // threads per workgroup (scan, draw)
constexpr int HT = 1024;         // threads per workgroup of the histogram passes
constexpr int kHistChunk = 4096; // vocabulary rows per histogram workgroup: every workgroup ends with up to
                                 // 256 atomic adds to memory per path, so few large ones are cheaper
constexpr int kBins = 256;       // 8 bits per level
constexpr int kLevels = 3;       // levels of the search: 24 key bits
constexpr float kMassScale = 17592186044416.0f;  // 2^44
constexpr int kNucBatch = 8;     // vocabulary rows a thread has in flight

__device__ __forceinline__ float nkey_logit(unsigned long long key) {
  uint32_t u = (uint32_t)(key >> 32);
  u = (u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u;
  return __uint_as_float(u);
}

// distance of a stored logit from its row's maximum in units of tau; the same expression in every pass
__device__ __forceinline__ float dist_t(float lmax, float l, float inv_tau) { return (lmax - l) * inv_tau; }

// The search key of t: t in units of 2^-19, saturated at 2^24 - 1.  (From t = 30.5 on, floor(e^-t * 2^44)
// is 0: whatever saturates carries no mass.)  Monotone in t, exact for the floats it is applied to.
__device__ __forceinline__ uint32_t order_key(float t) { return (uint32_t)fminf(t * 524288.0f, 16777215.0f); }

// floor(e^-t * 2^44).  The product is a float with 24 significant bits below 2^45, so it splits
// exactly into a multiple of 2^20 and a remainder below 2^20: two 32-bit conversions instead of the
// long software sequence of a float -> 64-bit integer conversion.
__device__ __forceinline__ unsigned long long mass_of(float t) {
  const float m = __builtin_amdgcn_exp2f(-t * 1.44269504088896341f) * kMassScale;
  const uint32_t hi = (uint32_t)(m * 9.5367431640625e-07f);        // m / 2^20, truncated
  const uint32_t lo = (uint32_t)(m - (float)hi * 1048576.0f);       // exact remainder
  return ((unsigned long long)hi << 20) + lo;
}

// LEVEL 0..2: digit = bits [23-8*LEVEL .. 16-8*LEVEL] of the key of t.
template <int LEVEL>
__global__ __launch_bounds__(HT) void nucleus_hist_kernel(const float* __restrict__ lt,
                                                          const unsigned long long* __restrict__ keys,
                                                          const uint32_t* __restrict__ prefix,
                                                          unsigned long long* __restrict__ ghist, NucGeom g,
                                                          float scale, float inv_tau) {
  extern __shared__ unsigned long long hist[];  // [KP][kBins]
  const int pos = blockIdx.x, c = blockIdx.y;
  const int tid = threadIdx.x;
  constexpr int shift = 8 * (kLevels - 1 - LEVEL);
  for (int x = tid; x < g.KP * kBins; x += HT) hist[x] = 0ull;
  __syncthreads();

  const int i = tid % g.KP;            // path of this thread (KP: K4 rounded up to a power of two, divides 256)
  const int vstep = HT / g.KP;         // vocabulary rows per sweep of the workgroup
  const bool live = i < g.KU;
  const int64_t row = (int64_t)pos * g.K + i;
  const float lmax = live ? scale * nkey_logit(keys[row]) : 0.f;
  const uint32_t pre = (LEVEL > 0 && live) ? prefix[row] : 0u;
  const float* base = lt + (int64_t)pos * g.V * g.K4 + i;
  const int v_end = min(g.V, (c + 1) * kHistChunk);
  if (live) {
    // the pass is bound by load latency unless many loads are in flight: kNucBatch rows are fetched
    // before the first is used (rows past the end re-read the last row and are skipped)
    for (int v0 = c * kHistChunk + tid / g.KP; v0 < v_end; v0 += kNucBatch * vstep) {
      float x[kNucBatch];
#pragma unroll
      for (int u = 0; u < kNucBatch; ++u) {
        const int v = v0 + u * vstep;
        x[u] = base[(int64_t)(v < v_end ? v : v_end - 1) * g.K4];
      }
      // LDS takes 64-bit atomics a lane at a time, so masses that fall into the bin of the element
      // before them (most do at the first level) are added up in registers first
      uint32_t run_bin = 0u;
      unsigned long long run_mass = 0ull;
#pragma unroll
      for (int u = 0; u < kNucBatch; ++u) {
        if (v0 + u * vstep >= v_end) break;
        const float t = dist_t(lmax, x[u], inv_tau);
        const uint32_t key = order_key(t);
        if (LEVEL > 0 && (key >> (shift + 8)) != (pre >> (shift + 8))) continue;
        const unsigned long long m = mass_of(t);
        const uint32_t bin = (key >> shift) & 255u;
        if (bin != run_bin && run_mass != 0ull) {
          atomicAdd(&hist[i * kBins + run_bin], run_mass);
          run_mass = 0ull;
        }
        run_bin = bin;
        run_mass += m;
      }
      if (run_mass != 0ull) atomicAdd(&hist[i * kBins + run_bin], run_mass);
    }
  }
  __syncthreads();
  for (int x = tid; x < g.KU * kBins; x += HT) {
    const unsigned long long m = hist[x];
    if (m != 0ull) atomicAdd(&ghist[((int64_t)pos * g.K + x / kBins) * kBins + (x % kBins)], m);
  }
}

// One wavefront per row: 4 consecutive bins per lane.
template <int LEVEL>
__global__ __launch_bounds__(NT) void nucleus_scan_kernel(unsigned long long* __restrict__ ghist,
                                                          uint32_t* __restrict__ prefix,
                                                          unsigned long long* __restrict__ below,
                                                          unsigned long long* __restrict__ target,
                                                          unsigned long long* __restrict__ keys_s, NucGeom g,
                                                          double top_p) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (NT / 64) + (threadIdx.x >> 6);
  if (row >= (int64_t)g.P * g.K) return;
  const int i = (int)(row % g.K);
  if (i >= g.KU) {  // the clean path draws nothing; its bins were never touched
    if (LEVEL == kLevels - 1 && lane == 0) keys_s[row] = 0ull;
    return;
  }
  constexpr int shift = 8 * (kLevels - 1 - LEVEL);
  unsigned long long* bins = ghist + row * kBins;
  unsigned long long b[4], run = 0ull;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    b[e] = bins[4 * lane + e];
    run += b[e];
    bins[4 * lane + e] = 0ull;  // ready for the next level (and for the next call)
  }
  // inclusive prefix sum of the lanes' totals over the wavefront
  unsigned long long incl = run;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long o = __shfl_up(incl, off, 64);
    if (lane >= off) incl += o;
  }
  const unsigned long long total = __shfl(incl, 63, 64);
  unsigned long long lo, want;
  if (LEVEL == 0) {
    lo = 0ull;
    // target = ceil(top_p * Z), never above Z and at least 1
    unsigned long long tg = (unsigned long long)ceil((double)total * top_p);
    tg = tg > total ? total : tg;
    want = tg < 1ull ? 1ull : tg;
  } else {
    lo = below[row];
    want = target[row];
  }
  // first bin at which lo + (mass of the bins up to and including it) reaches the target
  const bool mine = lo + incl >= want;
  const unsigned long long ballot = __ballot(mine);
  // by construction some bin reaches it; if rounding ever made none do, the last bin is taken
  const int first = ballot ? (int)__builtin_ctzll(ballot) : 63;
  if (lane == first) {
    unsigned long long acc = lo + (incl - run);
    int digit = 3;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (acc + b[e] >= want) {
        digit = e;
        break;
      }
      acc += b[e];
    }
    const uint32_t old = LEVEL == 0 ? 0u : prefix[row];
    prefix[row] = old | ((uint32_t)(4 * lane + digit) << shift);
    below[row] = acc;
    if (LEVEL == 0) target[row] = want;
    if (LEVEL == kLevels - 1) keys_s[row] = 0ull;
  }
}

// arg max of l / tau + noise over the nucleus; thread = (path, group of 4 consecutive vocabulary rows).
__global__ __launch_bounds__(NT) void nucleus_draw_kernel(const float* __restrict__ lt,
                                                          const unsigned long long* __restrict__ keys,
                                                          const uint32_t* __restrict__ thr,
                                                          unsigned long long* __restrict__ keys_s, NucGeom g,
                                                          SampleCfg samp, float scale, float inv_tau) {
  extern __shared__ unsigned long long red[];  // [KP][NT / KP]
  const int pos = blockIdx.x, c = blockIdx.y;
  const int tid = threadIdx.x;
  const int i = tid % g.KP;
  const int slot = tid / g.KP, nslot = NT / g.KP;
  const bool live = i < g.KU;
  const int64_t row = (int64_t)pos * g.K + i;
  unsigned long long best = 0ull;
  if (live) {
    const float lmax = scale * nkey_logit(keys[row]);
    const uint32_t tmax = thr[row];
    const RowRng rng = make_row_rng(samp, row, (int64_t)g.P * g.K);
    const float* base = lt + (int64_t)pos * g.V * g.K4 + i;
    const int v_end = min(g.V, (c + 1) * kNucChunk);
    constexpr int NB = 4;  // blocks of four rows in flight per thread
    for (int vb = c * kNucChunk + 4 * slot; vb < v_end; vb += NB * 4 * nslot) {
      float l[NB][4];
#pragma unroll
      for (int u = 0; u < NB; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = vb + u * 4 * nslot + e;
          l[u][e] = base[(int64_t)(v < v_end ? v : v_end - 1) * g.K4];
        }
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int v4 = vb + u * 4 * nslot;
        bool in[4];
        bool any = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          in[e] = v4 + e < v_end && order_key(dist_t(lmax, l[u][e], inv_tau)) <= tmax;
          any |= in[e];
        }
        if (!any) continue;
        float gn[4];
        gumbel4(rng, (uint32_t)v4, step_now(samp.step, samp.step_dev), gn);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (!in[e]) continue;
          const unsigned long long k = pack_key(fmaf(l[u][e], inv_tau, gn[e]) + 0.0f, (uint32_t)(v4 + e));
          best = k > best ? k : best;
        }
      }
    }
  } else if (i < g.K && slot == 0 && c == 0) {
    best = keys[row];  // the clean last path keeps its arg max
  }
  red[i * nslot + slot] = best;
  __syncthreads();
  if (tid < g.K) {
    unsigned long long k = 0ull;
    for (int s = 0; s < nslot; ++s) {
      const unsigned long long o = red[tid * nslot + s];
      k = o > k ? o : k;
    }
    if (k != 0ull) atomicMax(&keys_s[(int64_t)pos * g.K + tid], k);
  }
}

}  // namespace

hipError_t prepare_nucleus() {
  // the histograms of up to 64 paths need more LDS than the default limit
  hipError_t e;
  const int lds = kNucMaxK * kBins * 8;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(&nucleus_hist_kernel<0>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(&nucleus_hist_kernel<1>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds)) != hipSuccess) return e;
  static_assert(kLevels == 3, "one instance per level");
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&nucleus_hist_kernel<2>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

hipError_t launch_nucleus(const float* lt, const unsigned long long* keys, const NucBuffers& nb, const NucGeom& g,
                          const SampleCfg& samp, float scale, float inv_tau, double top_p, hipStream_t stream) {
  if (g.K < 1 || g.K > kNucMaxK || g.K4 < g.K || g.KP < g.K4 || (NT % g.KP) != 0 || g.KU < 1 || g.KU > g.K || g.P < 1 ||
      g.V < 1)
    return hipErrorInvalidValue;
  const int NC = (g.V + kNucChunk - 1) / kNucChunk;
  const int NH = (g.V + kHistChunk - 1) / kHistChunk;
  if (NC > 65535) return hipErrorInvalidValue;
  const dim3 grid((unsigned)g.P, (unsigned)NC), block(NT);
  const dim3 hgrid((unsigned)g.P, (unsigned)NH), hblock(HT);
  const size_t hist_lds = (size_t)g.KP * kBins * 8;
  const int64_t rows = (int64_t)g.P * g.K;
  const dim3 sgrid((unsigned)((rows + NT / 64 - 1) / (NT / 64)));
#define DM_NUC_LEVEL(L)                                                                                        \
  nucleus_hist_kernel<L><<<hgrid, hblock, hist_lds, stream>>>(lt, keys, nb.prefix, nb.hist, g, scale, inv_tau); \
  nucleus_scan_kernel<L><<<sgrid, block, 0, stream>>>(nb.hist, nb.prefix, nb.below, nb.target, nb.keys_s, g, top_p)
  DM_NUC_LEVEL(0);
  DM_NUC_LEVEL(1);
  DM_NUC_LEVEL(2);
#undef DM_NUC_LEVEL
  const size_t red_lds = (size_t)NT * 8;
  nucleus_draw_kernel<<<grid, block, red_lds, stream>>>(lt, keys, nb.prefix, nb.keys_s, g, samp, scale, inv_tau);
  return hipGetLastError();
}

}  // namespace dm
