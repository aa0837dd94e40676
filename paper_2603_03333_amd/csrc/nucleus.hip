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
// float32 logits are good for; tokens that share a key count as equally probable), 8 bits per level.
// Only the first level and the draw read the whole logit store:
//   nucleus_hist_kernel   per (position, chunk of vocabulary rows): the mass of every leading 8-bit
//                         digit - first in LDS (one histogram per path of the position), then the
//                         non-empty bins are added to the row's bins in memory (FINE: bins of two
//                         widths, see kFineShift below);
//   nucleus_scan_kernel   per row: walk the bins in order of growing t until the target mass
//                         ceil(top_p * Z) is reached: that is the BOUNDARY digit; the mass below it
//                         is carried on, the bins cleared for the next call;
//   nucleus_draw_kernel   every token with a smaller leading digit is in the nucleus whatever the
//                         other 16 bits of t* are: arg max of l[v] / tau + Gumbel noise over those
//                         (the same noise stream as the unrestricted draw, so top_p -> 1 gives that
//                         draw), merged into a second array of packed keys that the acceptance step
//                         reads; the tokens of the boundary digit (a few per cent of a row) are put
//                         on the row's candidate list, (logit, token) pairs, through LDS;
//   nucleus_finish_kernel per row: the two remaining levels of the search over the candidate list
//                         alone, then the draw among the candidates inside t*.  A row whose list
//                         did not fit (nearly uniform distributions: more than an eighth of the
//                         vocabulary shares the boundary digit) takes its candidates from the logit
//                         store instead.
// The first and third are bound by reading the logit store, 4 * K4 bytes per (position, vocabulary
// row) per pass, and by the vector ALU (t, key, integer mass; the noise of half the vocabulary).
#include "kernels.hpp"
#include "sampling.hpp"

namespace dm {
namespace {

constexpr int NT = 256;          // threads per workgroup (scan, draw)
constexpr int HT = 1024;         // threads per workgroup of the histogram pass
constexpr int kHistChunk = 4096; // vocabulary rows per histogram workgroup: every workgroup ends with up to
                                 // 256 atomic adds to memory per path, so few large ones are cheaper
constexpr int kBins = 256;       // 8 bits per level
// The first histogram has bins of two widths, so that a very flat row (most of its tokens within a fraction
// of the maximum) does not put the whole vocabulary into one bin: keys below 2^20 (t < 2) go by their FINE
// digit key >> 12 (t in steps of 1/128, slots 0..255), the others by their COARSE digit key >> 16 (steps
// of 1/8 up to 32; digits 16..255 in slots 256..495).  Every element adds to exactly one slot.
constexpr int kCoarseShift = 16;
constexpr int kFineShift = 12;
constexpr uint32_t kFineLimit = 1u << (kFineShift + 8);                 // keys that have a fine digit
constexpr uint32_t kCoarseFirst = kFineLimit >> kCoarseShift;           // 16: the first coarse digit with a slot of its own
constexpr uint32_t kCoarseSlot0 = kBins - kCoarseFirst;                 // slot of coarse digit c: kCoarseSlot0 + c
constexpr int kLevels = 3;       // levels of the search: 24 key bits
constexpr float kMassScale = 17592186044416.0f;  // 2^44
constexpr int kNucBatch = 8;     // vocabulary rows a thread has in flight
constexpr int FT = 512;          // threads per workgroup of the finishing pass
constexpr int kNucStage = 128;   // candidates per path that a draw workgroup can stage in LDS (an eighth of its rows)
constexpr uint32_t kNoToken = 0xFFFFFFFFu;   // no token (never a valid one: V < 2^31)
constexpr uint32_t kNucNoFit = 0x80000000u;  // set in a list's count by a workgroup whose stage ran over

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

// The coarse digit straight from t: order_key(t) >> 16 (scaling by a power of two is exact and
// floor(floor(x) / 2^16) = floor(x / 2^16)).
__device__ __forceinline__ uint32_t coarse_digit(float t) { return (uint32_t)fminf(t * 8.0f, 255.0f); }

// floor(e^-t * 2^44).  The product is a float with 24 significant bits below 2^45, so it splits
// exactly into a multiple of 2^20 and a remainder below 2^20: two 32-bit conversions instead of the
// long software sequence of a float -> 64-bit integer conversion.
__device__ __forceinline__ unsigned long long mass_of(float t) {
  const float m = __builtin_amdgcn_exp2f(-t * 1.44269504088896341f) * kMassScale;
  const uint32_t hi = (uint32_t)(m * 9.5367431640625e-07f);        // m / 2^20, truncated
  const uint32_t lo = (uint32_t)(m - (float)hi * 1048576.0f);       // exact remainder, below 2^20
  // hi * 2^20 + lo as a pair of 32-bit words (two plain instructions; the 64-bit shift and add cost six issue slots)
  return ((unsigned long long)(hi >> 12) << 32) | (unsigned long long)((hi << 20) | lo);
}

// The mass of every element of the chunk, by its leading digit (coarse, or FINE: of either width).
template <bool FINE>
__global__ __launch_bounds__(HT) void nucleus_hist_kernel(const float* __restrict__ lt,
                                                          const unsigned long long* __restrict__ keys,
                                                          unsigned long long* __restrict__ ghist, NucGeom g,
                                                          float scale, float inv_tau) {
  extern __shared__ unsigned long long hist[];  // [KP][bins]: FINE: 256 fine + 240 coarse slots; else 256 coarse digits
  const int pos = blockIdx.x, c = blockIdx.y;
  const int tid = threadIdx.x;
  constexpr int bins = FINE ? 2 * kBins : kBins;
  for (int x = tid; x < g.KP * bins; x += HT) hist[x] = 0ull;
  __syncthreads();

  // thread = four paths (one 16-byte piece of a store row) x every (HT / KQ)-th vocabulary row
  const int KQ = g.KP / 4;
  const int q = tid % KQ;
  const int vstep = HT / KQ;           // vocabulary rows per sweep of the workgroup
  float lmax[4];
  bool live[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    live[j] = 4 * q + j < g.KU;
    lmax[j] = live[j] ? scale * nkey_logit(keys[(int64_t)pos * g.K + 4 * q + j]) : 0.f;
  }
  const float* base = lt + (int64_t)pos * g.V * g.K4 + 4 * q;
  const int v_end = min(g.V, (c + 1) * kHistChunk);
  if (4 * q < g.K4) {
    // kNucBatch rows (16 bytes of each) are in flight before the first is used; rows past the end re-read
    // the last row and are skipped
    for (int v0 = c * kHistChunk + tid / KQ; v0 < v_end; v0 += kNucBatch * vstep) {
      float4 x[kNucBatch];
#pragma unroll
      for (int u = 0; u < kNucBatch; ++u) {
        const int v = v0 + u * vstep;
        x[u] = *reinterpret_cast<const float4*>(base + (int64_t)(v < v_end ? v : v_end - 1) * g.K4);
      }
      // one LDS atomic per element: adding up runs of equal digits in registers first costs more vector
      // instructions than the atomics it saves (the pass is bound by the vector ALU, then by these atomics)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (!live[j]) continue;
        unsigned long long* hj = hist + (4 * q + j) * bins;
#pragma unroll
        for (int u = 0; u < kNucBatch; ++u) {
          const float xu = j == 0 ? x[u].x : j == 1 ? x[u].y : j == 2 ? x[u].z : x[u].w;
          const float t = dist_t(lmax[j], xu, inv_tau);
          const unsigned long long m = mass_of(t);
          uint32_t slot;
          if constexpr (FINE) {
            const uint32_t key = order_key(t);
            slot = key < kFineLimit ? key >> kFineShift : kCoarseSlot0 + (key >> kCoarseShift);
          } else {
            slot = coarse_digit(t);
          }
          if (v0 + u * vstep < v_end) atomicAdd(&hj[slot], m);
        }
      }
    }
  }
  __syncthreads();
  for (int x = tid; x < g.KU * bins; x += HT) {
    const unsigned long long m = hist[x];
    if (m != 0ull) atomicAdd(&ghist[((int64_t)pos * g.K + x / bins) * (2 * kBins) + (x % bins)], m);
  }
}

// One level of the search, by one wavefront: lane l holds bins 4l .. 4l+3 (b) of 256; lo = mass below the
// digits fixed so far, want = mass to reach.  Returns the first bin at which lo + (mass of the bins up to and
// including it) reaches want, and in lo the mass below that bin.  (Some bin reaches it by construction; if
// rounding ever made none do, the last bin is taken.)
__device__ __forceinline__ int search_bins(const unsigned long long (&b)[4], unsigned long long& lo,
                                           unsigned long long want) {
  const int lane = threadIdx.x & 63;
  const unsigned long long run = b[0] + b[1] + b[2] + b[3];
  unsigned long long incl = run;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long o = __shfl_up(incl, off, 64);
    if (lane >= off) incl += o;
  }
  const unsigned long long ballot = __ballot(lo + incl >= want);
  const int first = ballot ? (int)__builtin_ctzll(ballot) : 63;
  unsigned long long acc = lo + (incl - run);
  int digit = 3;
  bool found = false;
#pragma unroll
  for (int e = 0; e < 3; ++e) {
    if (!found && acc + b[e] >= want) {
      digit = e;
      found = true;
    }
    if (!found) acc += b[e];
  }
  lo = __shfl(acc, first, 64);
  return 4 * first + __shfl(digit, first, 64);
}

// First level, one wavefront per row.  Also turns top_p into the target mass and readies the row's
// per-call state: bins cleared, candidate list empty, no drawn token yet.
__global__ __launch_bounds__(NT) void nucleus_scan_kernel(unsigned long long* __restrict__ ghist,
                                                          uint32_t* __restrict__ digit0,
                                                          unsigned long long* __restrict__ below,
                                                          unsigned long long* __restrict__ target,
                                                          uint32_t* __restrict__ cand_n,
                                                          unsigned long long* __restrict__ keys_s, NucGeom g,
                                                          double top_p) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (NT / 64) + (threadIdx.x >> 6);
  if (row >= (int64_t)g.P * g.K) return;
  const int i = (int)(row % g.K);
  if (lane == 0) {
    keys_s[row] = 0ull;
    cand_n[row] = 0u;
  }
  if (i >= g.KU) return;  // the clean path draws nothing; its bins were never touched
  // slots 0..255 (fine digits, or all 256 coarse digits without the fine bins), then slots 256..511
  unsigned long long* bins = ghist + row * (2 * kBins);
  unsigned long long b[4], b2[4], first_half = 0ull, second_half = 0ull;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    b[e] = bins[4 * lane + e];
    first_half += b[e];
    bins[4 * lane + e] = 0ull;
    b2[e] = 0ull;
    if (g.fine) {
      b2[e] = bins[kBins + 4 * lane + e];
      second_half += b2[e];
      bins[kBins + 4 * lane + e] = 0ull;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    first_half += __shfl_xor(first_half, off, 64);
    second_half += __shfl_xor(second_half, off, 64);
  }
  const unsigned long long total = first_half + second_half;
  // target = ceil(top_p * Z), never above Z and at least 1
  unsigned long long want = (unsigned long long)ceil((double)total * top_p);
  want = want > total ? total : want;
  want = want < 1ull ? 1ull : want;
  unsigned long long lo = 0ull;
  int digit, shift;
  if (!g.fine) {
    digit = search_bins(b, lo, want);
    shift = kCoarseShift;
  } else if (want <= first_half) {  // the threshold lies within 2 of the row's maximum: a fine digit
    digit = search_bins(b, lo, want);
    shift = kFineShift;
  } else {
    lo = first_half;
    digit = search_bins(b2, lo, want) + (int)kCoarseFirst;
    shift = kCoarseShift;
  }
  if (lane == 0) {
    digit0[row] = (uint32_t)digit | ((uint32_t)shift << 16);
    below[row] = lo;
    target[row] = want;
  }
}

// arg max of l / tau + noise over the tokens whose leading digit lies below the boundary digit, and the
// tokens of the boundary digit onto the candidate list; thread = (path, group of 4 consecutive vocabulary
// rows = one block of the noise stream).
template <bool FINE>
__global__ __launch_bounds__(NT) void nucleus_draw_kernel(const float* __restrict__ lt,
                                                          const unsigned long long* __restrict__ keys,
                                                          const uint32_t* __restrict__ digit0,
                                                          unsigned long long* __restrict__ keys_s,
                                                          uint2* __restrict__ cand, uint32_t* __restrict__ cand_n,
                                                          NucGeom g, SampleCfg samp, float scale, float inv_tau) {
  extern __shared__ unsigned long long red[];  // [KP][NT / KP] keys, then [KP][wcap] staged candidates
  __shared__ uint32_t cnt[kNucMaxK], dst0[kNucMaxK];
  const int pos = blockIdx.x, c = blockIdx.y;
  const int tid = threadIdx.x;
  const int i = tid % g.KP;
  const int slot = tid / g.KP, nslot = NT / g.KP;
  constexpr int wcap = kNucStage;      // staged candidates per path
  uint2* stage = reinterpret_cast<uint2*>(red + NT);
  const bool live = i < g.KU;
  const int64_t row = (int64_t)pos * g.K + i;
  if (tid < kNucMaxK) cnt[tid] = 0u;
  __syncthreads();
  unsigned long long best = 0ull;
  if (live) {
    const float lmax = scale * nkey_logit(keys[row]);
    const uint32_t d0 = digit0[row] & 0xFFFFu, sh0 = digit0[row] >> 16;  // boundary digit and where it sits in the key
    const RowRng rng = make_row_rng(samp, row, (int64_t)g.P * g.K);
    const uint32_t step = step_now(samp.step, samp.step_dev);
    const float* base = lt + (int64_t)pos * g.V * g.K4 + i;
    const int v_end = min(g.V, (c + 1) * kNucChunk);
    constexpr int NB = 4;  // blocks of four rows in flight per thread
    // the running best as (value, token): a thread meets its tokens in growing order, so among equal values
    // the first one met is the smaller token, as in the packed keys
    float best_y = -INFINITY;
    uint32_t best_v = kNoToken;
    for (int vb = c * kNucChunk + 4 * slot; vb < v_end; vb += NB * 4 * nslot) {
      const bool whole = vb + (NB - 1) * 4 * nslot + 3 < v_end;  // all NB blocks inside the chunk
      float l[NB][4];
#pragma unroll
      for (int u = 0; u < NB; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = vb + u * 4 * nslot + e;
          // offsets inside one position's part of the store fit 32 bits (checked by the caller)
          l[u][e] = base[(uint32_t)((whole || v < v_end) ? v : v_end - 1) * (uint32_t)g.K4];
        }
      uint32_t in = 0u, cd = 0u;  // bit 4u + e: token inside for sure / candidate
#pragma unroll
      for (int u = 0; u < NB; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float t = dist_t(lmax, l[u][e], inv_tau);
          const uint32_t dg = FINE ? order_key(t) >> sh0 : coarse_digit(t);  // not FINE: sh0 is 16 for every row
          const bool there = whole || vb + u * 4 * nslot + e < v_end;
          in |= (there && dg < d0) ? 1u << (4 * u + e) : 0u;
          cd |= (there && dg == d0) ? 1u << (4 * u + e) : 0u;
        }
      if (cd != 0u) {  // room for all of them with one atomic, then plain writes
        uint32_t at = atomicAdd(&cnt[i], (uint32_t)__popc(cd));
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (cd & (1u << (4 * u + e))) {
              if (at < (uint32_t)wcap)
                stage[i * wcap + at] = make_uint2(__float_as_uint(l[u][e]), (uint32_t)(vb + u * 4 * nslot + e));
              ++at;
            }
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        if (((in >> (4 * u)) & 15u) == 0u) continue;
        const int v4 = vb + u * 4 * nslot;
        float gn[4];
        gumbel4(rng, (uint32_t)v4, step, gn);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float y = fmaf(l[u][e], inv_tau, gn[e]);
          const bool take = (in & (1u << (4 * u + e))) && y > best_y;
          best_y = take ? y : best_y;
          best_v = take ? (uint32_t)(v4 + e) : best_v;
        }
      }
    }
    if (best_v != kNoToken) best = pack_key(best_y + 0.0f, best_v);
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
    // room on the row's list for this workgroup's candidates; a workgroup whose stage ran over marks the list
    // as not fitting (top bit of the count, which the additions never reach: they sum to at most V), and a
    // list that runs over shows in the count itself
    const uint32_t n = tid < g.KU ? cnt[tid] : 0u;
    if (n > (uint32_t)wcap)
      atomicOr(&cand_n[(int64_t)pos * g.K + tid], kNucNoFit);
    else if (n != 0u)
      dst0[tid] = atomicAdd(&cand_n[(int64_t)pos * g.K + tid], n);
  }
  __syncthreads();
  for (int x = tid; x < g.KP * wcap; x += NT) {
    const int pi = x / wcap, xi = x - pi * wcap;
    if (pi >= g.KU) break;
    const uint32_t n = cnt[pi];
    if (n > (uint32_t)wcap || (uint32_t)xi >= n) continue;
    const uint64_t at = (uint64_t)dst0[pi] + (uint32_t)xi;
    if (at < (uint64_t)g.cap) cand[((int64_t)pos * g.K + pi) * g.cap + (int64_t)at] = stage[x];
  }
}


// The candidates of one row: in registers (lists of up to EPT * FT entries, read once: every list of a flat
// Gaussian row at the sizes of the benchmark), from the list in memory (longer ones), or - the list did not
// fit - from the logit store.  Calls f(logit, token) for the candidates of every `every`-th round of the
// workgroup's threads striding over them, starting with round `first`.
constexpr int EPT = 8;
template <typename F>
__device__ __forceinline__ void for_candidates(bool in_regs, const uint2 (&held)[EPT], bool fits,
                                               const uint2* __restrict__ list, uint32_t n,
                                               const float* __restrict__ col, int V, int K4, float lmax, float inv_tau,
                                               uint32_t d0, uint32_t sh0, int first, int every, F f) {
  if (in_regs) {
#pragma unroll
    for (int u = 0; u < EPT; ++u)
      if (held[u].y != kNoToken && (every == 1 || u % every == first)) f(__uint_as_float(held[u].x), held[u].y);
  } else if (fits) {
    for (uint32_t x = threadIdx.x + (uint32_t)first * FT; x < n; x += (uint32_t)every * FT) {
      const uint2 e = list[x];
      f(__uint_as_float(e.x), e.y);
    }
  } else {
    for (int64_t v = threadIdx.x + (int64_t)first * FT; v < V; v += (int64_t)every * FT) {
      const float l = col[v * K4];
      if ((order_key(dist_t(lmax, l, inv_tau)) >> sh0) == d0) f(l, (uint32_t)v);
    }
  }
}

// Levels two and three of the search and the draw among the candidates.  gridDim.y workgroups per row: each
// settles the threshold for itself (a few thousand candidates) and draws among its share of them - the noise
// of a candidate costs far more than its part in the search, and few rows would otherwise keep few compute
// units busy.
__global__ __launch_bounds__(FT) void nucleus_finish_kernel(const float* __restrict__ lt,
                                                            const unsigned long long* __restrict__ keys,
                                                            const uint32_t* __restrict__ digit0,
                                                            const unsigned long long* __restrict__ below,
                                                            const unsigned long long* __restrict__ target,
                                                            const uint2* __restrict__ cand,
                                                            const uint32_t* __restrict__ cand_n,
                                                            unsigned long long* __restrict__ keys_s, NucGeom g,
                                                            SampleCfg samp, float scale, float inv_tau) {
  __shared__ unsigned long long hist[kLevels - 1][kBins];
  __shared__ unsigned long long best_s[FT / 64];
  const int64_t row = blockIdx.x;
  const int pos = (int)(row / g.K), i = (int)(row % g.K);
  if (i >= g.KU) return;
  const int tid = threadIdx.x, lane = tid & 63;
  // the head of the list is fetched before its length is known (one round trip to memory instead of two);
  // what lies beyond the length is dropped afterwards
  const uint2* list = cand + row * g.cap;
  uint2 held[EPT];
#pragma unroll
  for (int u = 0; u < EPT; ++u) {
    const uint32_t x = (uint32_t)tid + (uint32_t)u * FT;
    held[u] = x < (uint32_t)g.cap ? list[x] : make_uint2(0u, kNoToken);
  }
  const uint32_t n = cand_n[row];
  const bool fits = n <= (uint32_t)g.cap;
  const bool in_regs = n <= (uint32_t)(EPT * FT) && fits;
#pragma unroll
  for (int u = 0; u < EPT; ++u)
    if (!in_regs || (uint32_t)tid + (uint32_t)u * FT >= n) held[u].y = kNoToken;
  const float* col = lt + (int64_t)pos * g.V * g.K4 + i;
  const float lmax = scale * nkey_logit(keys[row]);
  const uint32_t d0 = digit0[row] & 0xFFFFu, sh0 = digit0[row] >> 16;
  const unsigned long long want = target[row];
  unsigned long long lo = below[row];
  for (int x = tid; x < (kLevels - 1) * kBins; x += FT) hist[0][x] = 0ull;
  __syncthreads();
  // the remaining sh0 bits of the key, up to 8 at a time (16 = 8 + 8 below a coarse digit, 12 = 8 + 4 below a fine one)
  uint32_t thr = d0 << sh0;
  int shift = (int)sh0;
#pragma unroll
  for (int level = 1; level < kLevels; ++level) {
    const int nb = shift > 8 ? 8 : shift;
    shift -= nb;
    const uint32_t digit_mask = (1u << nb) - 1u;
    unsigned long long* hl = hist[level - 1];
    for_candidates(in_regs, held, fits, list, n, col, g.V, g.K4, lmax, inv_tau, d0, sh0, 0, 1, [&](float l, uint32_t) {
      const float t = dist_t(lmax, l, inv_tau);
      const uint32_t key = order_key(t);
      if ((key >> (shift + nb)) == (thr >> (shift + nb))) atomicAdd(&hl[(key >> shift) & digit_mask], mass_of(t));
    });
    __syncthreads();
    // every wavefront walks the bins for itself: no second barrier, nothing to hand round
    unsigned long long b[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) b[e] = hl[4 * lane + e];
    thr |= (uint32_t)search_bins(b, lo, want) << shift;
  }
  // the draw among the candidates inside the threshold
  const RowRng rng = make_row_rng(samp, row, (int64_t)g.P * g.K);
  const uint32_t step = step_now(samp.step, samp.step_dev);
  unsigned long long best = 0ull;
  const int share = blockIdx.y, shares = gridDim.y;  // shares: a power of two up to EPT
  for_candidates(in_regs, held, fits, list, n, col, g.V, g.K4, lmax, inv_tau, d0, sh0, share, shares, [&](float l, uint32_t v) {
    if (order_key(dist_t(lmax, l, inv_tau)) > thr) return;
    float gn[4];
    gumbel4(rng, v & ~3u, step, gn);
    const float noise = (v & 2u) ? ((v & 1u) ? gn[3] : gn[2]) : ((v & 1u) ? gn[1] : gn[0]);
    const unsigned long long k = pack_key(fmaf(l, inv_tau, noise) + 0.0f, v);
    best = k > best ? k : best;
  });
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(best, off, 64);
    best = o > best ? o : best;
  }
  if (lane == 0) best_s[tid >> 6] = best;
  __syncthreads();
  if (tid == 0) {
    unsigned long long k = 0ull;
    for (int w = 0; w < FT / 64; ++w) k = best_s[w] > k ? best_s[w] : k;
    // merged with what the draw pass found among the tokens below the boundary digit
    if (k != 0ull) atomicMax(&keys_s[row], k);
  }
}

}  // namespace

hipError_t prepare_nucleus() {
  // the histograms of up to 64 paths (32 with the fine bins) need more LDS than the default limit
  hipError_t e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(&nucleus_hist_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kNucMaxK * kBins * 8)) != hipSuccess ||
      (e = hipFuncSetAttribute(reinterpret_cast<const void*>(&nucleus_hist_kernel<true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kNucFineMaxKP * 2 * kBins * 8)) != hipSuccess ||
      (e = hipFuncSetAttribute(reinterpret_cast<const void*>(&nucleus_draw_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, NT * 8 + kNucMaxK * kNucStage * 8)) != hipSuccess)
    return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&nucleus_draw_kernel<true>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, NT * 8 + kNucMaxK * kNucStage * 8);
}

hipError_t launch_nucleus(const float* lt, const unsigned long long* keys, const NucBuffers& nb, const NucGeom& g,
                          const SampleCfg& samp, float scale, float inv_tau, double top_p, hipStream_t stream) {
  if (g.K < 1 || g.K > kNucMaxK || g.K4 < g.K || g.KP < g.K4 || (NT % g.KP) != 0 || g.KU < 1 || g.KU > g.K || g.P < 1 ||
      g.V < 1 || g.cap < 1 || (int64_t)g.P * g.K > 0x7FFFFFFF)
    return hipErrorInvalidValue;
  const int NC = (g.V + kNucChunk - 1) / kNucChunk;
  const int NH = (g.V + kHistChunk - 1) / kHistChunk;
  if (NC > 65535) return hipErrorInvalidValue;
  const dim3 grid((unsigned)g.P, (unsigned)NC), block(NT);
  const dim3 hgrid((unsigned)g.P, (unsigned)NH), hblock(HT);
  const int64_t rows = (int64_t)g.P * g.K;
  const dim3 sgrid((unsigned)((rows + NT / 64 - 1) / (NT / 64)));
  if (g.fine && g.KP > kNucFineMaxKP) return hipErrorInvalidValue;
  if (g.fine)
    nucleus_hist_kernel<true><<<hgrid, hblock, (size_t)g.KP * 2 * kBins * 8, stream>>>(lt, keys, nb.hist, g, scale, inv_tau);
  else
    nucleus_hist_kernel<false><<<hgrid, hblock, (size_t)g.KP * kBins * 8, stream>>>(lt, keys, nb.hist, g, scale, inv_tau);
  nucleus_scan_kernel<<<sgrid, block, 0, stream>>>(nb.hist, nb.digit0, nb.below, nb.target, nb.cand_n, nb.keys_s, g, top_p);
  const size_t draw_lds = (size_t)NT * 8 + (size_t)g.KP * kNucStage * 8;
  if (g.fine)
    nucleus_draw_kernel<true><<<grid, block, draw_lds, stream>>>(lt, keys, nb.digit0, nb.keys_s, nb.cand, nb.cand_n, g, samp,
                                                                scale, inv_tau);
  else
    nucleus_draw_kernel<false><<<grid, block, draw_lds, stream>>>(lt, keys, nb.digit0, nb.keys_s, nb.cand, nb.cand_n, g, samp,
                                                                 scale, inv_tau);
  unsigned shares = 1;  // workgroups per row of the last pass: as many as it takes to use the chip, at most EPT
  while (shares < (unsigned)EPT && rows * shares < 512) shares *= 2;
  nucleus_finish_kernel<<<dim3((unsigned)rows, shares), dim3(FT), 0, stream>>>(lt, keys, nb.digit0, nb.below, nb.target, nb.cand,
                                                                      nb.cand_n, nb.keys_s, g, samp, scale, inv_tau);
  return hipGetLastError();
}

}  // namespace dm
