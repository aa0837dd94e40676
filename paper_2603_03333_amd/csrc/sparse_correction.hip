// The same path logits by linearity (Eq. (2)-(3)):  W (h * m) = W h - W (h * (1 - m)).
// One clean row per position (the plain LM head, on the matrix cores, 1/K of the dense work) and, per
// path, a correction over the dimensions that path DROPPED (a fraction p of d).  The dropped dimensions
// differ from path to path, and an MFMA tile needs all its rows to share their k indices, so the
// corrections cannot run on the matrix cores as they are; here they run on the vector ALU.  (The 2:4
// structured-sparsity MFMA does not fit either: a group of four dimensions holds three or four dropped
// ones with probability 0.37 % at p = 0.1, seven to eight such groups per row at d = 8192, and an exact
// result would need those handled beside the matrix instruction for every vocabulary row.)
// This file is the measured answer to "does that pay on this chip": the vector ALU does one
// multiply-add per lane and cycle where the matrix cores do sixteen, so at p = 0.1 the corrections
// alone cost more than the whole dense contraction.  Kept as an option (DM_FLAG_SPARSE_CORRECTION),
// parity-tested, not used by default.
//
//   drop_lists_kernel      per masked row and k slab of 64: the dropped dimensions (from the same
//                          Philox stream as the masks of Eq. (1)) with their h values, compacted.
//   sparse_correct_kernel  workgroup = 64 vocabulary rows x 4 positions; the W slab goes through LDS
//                          (rows padded to 33 words: a column read is conflict-free) together with the
//                          lists of the slab, every thread owns one vocabulary row of one position and
//                          the K running corrections of its paths; the lists are uniform over a
//                          wavefront.  At the end logit = clean - correction, wavefront arg max,
//                          packed-key atomicMax.
#include "kernels.hpp"
#include "philox.hpp"

namespace dm {
namespace {

constexpr int SK = 64;        // k per slab
constexpr int SV = 64;        // vocabulary rows per workgroup
constexpr int SP = 4;         // positions per workgroup
constexpr int ROW_WORDS = 33; // 64 bf16 = 32 words, + 1 word of padding

__global__ __launch_bounds__(256) void drop_lists_kernel(const uint16_t* __restrict__ h, uint32_t* __restrict__ ent,
                                                         uint32_t* __restrict__ cnt,
                                                         unsigned long long* __restrict__ keys, SeedPack seeds,
                                                         RowGeom g, int64_t row0, int64_t nrows, int b0) {
  const int lane = threadIdx.x & 63;
  const int64_t r = row0 + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= row0 + nrows) return;
  const int TK = g.T * g.K;
  const int b = (int)(r / TK);
  const int rem = (int)(r - (int64_t)b * TK);
  const int t = rem / g.K;
  const int i = rem - t * g.K;
  const uint64_t seed = seeds.s[b - b0];
  const bool clean = g.clean_last && i == g.K - 1;
  const int nslab = g.d / SK;
  const uint16_t* hrow = h + ((int64_t)b * g.T + t) * g.d;
  if (lane == 0) keys[r] = 0ull;
  for (int s = 0; s < nslab; ++s) {
    const int j = s * SK + lane;
    const uint32_t bits = keep_bits8((uint32_t)j >> 3, g.share_pos ? 0u : (uint32_t)t, (uint32_t)i, step_now(g.step, g.step_dev),
                                     (uint32_t)seed, (uint32_t)(seed >> 32), g.thr);
    const bool dropped = !clean && ((bits >> (j & 7)) & 1u) == 0u;
    const unsigned long long m = __ballot(dropped);
    const int at = __popcll(m & ((1ull << lane) - 1ull));
    if (dropped) ent[(r * nslab + s) * SK + at] = (uint32_t)lane | ((uint32_t)hrow[j] << 16);
    if (lane == 0) cnt[r * nslab + s] = (uint32_t)__popcll(m);
  }
}

constexpr int LCAP = 16;      // entries of a list that travel through LDS with the slab (the rest, rare, from memory)

template <int KMAX>
__global__ __launch_bounds__(256) void sparse_correct_kernel(const uint16_t* __restrict__ W,
                                                             const float* __restrict__ clean,
                                                             const uint32_t* __restrict__ ent,
                                                             const uint32_t* __restrict__ cnt,
                                                             unsigned long long* __restrict__ keys, int P, int K,
                                                             int d, int V) {
  __shared__ uint32_t ws[SV * ROW_WORDS];          // the W slab
  __shared__ uint32_t ls_ent[SP * KMAX * LCAP];    // first LCAP entries of every list of the slab
  __shared__ uint32_t ls_cnt[SP * KMAX];
  const int tid = threadIdx.x;
  const int vl = tid & 63, pl = tid >> 6;
  const int v0 = blockIdx.x * SV;
  const int pos0 = blockIdx.y * SP;
  const int pos = pos0 + pl;
  const bool pos_ok = pos < P;
  const int nslab = d / SK;
  float acc[KMAX];
#pragma unroll
  for (int i = 0; i < KMAX; ++i) acc[i] = 0.f;

  // loader roles: W row tid / 4 of the slab, 16 elements (32 bytes) starting at (tid % 4) * 16;
  // list words: thread x takes word x % LCAP of list x / LCAP, SP * KMAX lists in all
  const int lr = tid >> 2, lq = tid & 3;
  const int lrow = (v0 + lr < V) ? v0 + lr : V - 1;
  const uint4* lsrc = reinterpret_cast<const uint4*>(W + (int64_t)lrow * d) + lq * 2;
  for (int s = 0; s < nslab; ++s) {
    const uint4 a = lsrc[s * 8], b = lsrc[s * 8 + 1];
    uint32_t lw[(SP * KMAX * LCAP + 255) / 256];
    uint32_t lc = 0u;
#pragma unroll
    for (int u = 0; u < (SP * KMAX * LCAP + 255) / 256; ++u) {
      const int x = tid + 256 * u;
      const int list = x / LCAP, word = x % LCAP;
      const int lp = list / KMAX, li = list % KMAX;
      const bool on = list < SP * KMAX && pos0 + lp < P && li < K;
      lw[u] = on ? ent[(((int64_t)(pos0 + lp) * K + li) * nslab + s) * SK + word] : 0u;
    }
    if (tid < SP * KMAX) {
      const int lp = tid / KMAX, li = tid % KMAX;
      lc = (pos0 + lp < P && li < K) ? cnt[((int64_t)(pos0 + lp) * K + li) * nslab + s] : 0u;
    }
    __syncthreads();  // the slab before has been used by everybody
    uint32_t* dst = ws + lr * ROW_WORDS + lq * 8;
    dst[0] = a.x; dst[1] = a.y; dst[2] = a.z; dst[3] = a.w;
    dst[4] = b.x; dst[5] = b.y; dst[6] = b.z; dst[7] = b.w;
#pragma unroll
    for (int u = 0; u < (SP * KMAX * LCAP + 255) / 256; ++u)
      if (tid + 256 * u < SP * KMAX * LCAP) ls_ent[tid + 256 * u] = lw[u];
    if (tid < SP * KMAX) ls_cnt[tid] = lc;
    __syncthreads();
    if (pos_ok) {
      const uint32_t* wrow = ws + vl * ROW_WORDS;
#pragma unroll
      for (int i = 0; i < KMAX; ++i) {
        if (i < K) {
          const int n = (int)ls_cnt[pl * KMAX + i];        // uniform over the wavefront
          const uint32_t* e = ls_ent + (pl * KMAX + i) * LCAP;
          const int n_lds = n < LCAP ? n : LCAP;
          for (int x = 0; x < n_lds; ++x) {
            const uint32_t word = e[x];
            const uint32_t j = word & 63u;
            const uint32_t w2 = wrow[j >> 1];
            const float w = __uint_as_float((j & 1u) ? (w2 & 0xFFFF0000u) : (w2 << 16));
            acc[i] = fmaf(w, __uint_as_float(word & 0xFFFF0000u), acc[i]);
          }
          if (n > LCAP) {  // a long list (rare unless p is large): the rest from memory
            const uint32_t* eg = ent + (((int64_t)pos * K + i) * nslab + s) * SK;
            for (int x = LCAP; x < n; ++x) {
              const uint32_t word = eg[x];
              const uint32_t j = word & 63u;
              const uint32_t w2 = wrow[j >> 1];
              const float w = __uint_as_float((j & 1u) ? (w2 & 0xFFFF0000u) : (w2 << 16));
              acc[i] = fmaf(w, __uint_as_float(word & 0xFFFF0000u), acc[i]);
            }
          }
        }
      }
    }
  }
  // logit = clean - correction; arg max over the 64 vocabulary rows of the wavefront, then over the launch
  const int v = v0 + vl;
  const bool ok = pos_ok && v < V;
  const float c = ok ? clean[(int64_t)pos * V + v] : 0.f;
#pragma unroll
  for (int i = 0; i < KMAX; ++i) {
    if (i < K) {
      unsigned long long key = ok ? pack_key((c - acc[i]) + 0.0f, (uint32_t)v) : 0ull;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(key, off, 64);
        key = o > key ? o : key;
      }
      if (vl == 0 && pos_ok && key != 0ull) atomicMax(&keys[(int64_t)pos * K + i], key);
    }
  }
}

}  // namespace

hipError_t launch_drop_lists(const void* h, uint32_t* ent, uint32_t* cnt, unsigned long long* keys,
                             const uint64_t* seeds_host, const RowGeom& g, hipStream_t stream) {
  if (g.d % SK != 0) return hipErrorInvalidValue;
  const int64_t TK = (int64_t)g.T * g.K;
  for (int b0 = 0; b0 < g.B; b0 += kSeedsPerLaunch) {
    const int nb = (g.B - b0 < kSeedsPerLaunch) ? (g.B - b0) : kSeedsPerLaunch;
    SeedPack sp;
    for (int q = 0; q < kSeedsPerLaunch; ++q) sp.s[q] = (q < nb) ? seeds_host[b0 + q] : 0ull;
    const int64_t row0 = (int64_t)b0 * TK, nrows = (int64_t)nb * TK;
    const int64_t nblocks = (nrows + 3) / 4;
    if (nblocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    drop_lists_kernel<<<dim3((unsigned)nblocks), dim3(256), 0, stream>>>(static_cast<const uint16_t*>(h), ent, cnt, keys,
                                                                        sp, g, row0, nrows, b0);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_sparse_correct(const void* W, const float* clean, const uint32_t* ent, const uint32_t* cnt,
                                 unsigned long long* keys, int P, int K, int d, int V, hipStream_t stream) {
  if (K < 1 || K > kSparseMaxK || d % SK != 0 || P < 1 || V < 1) return hipErrorInvalidValue;
  const unsigned gy = (unsigned)((P + SP - 1) / SP);
  if (gy > 65535u) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((V + SV - 1) / SV), gy), block(256);
  if (K <= 8)
    sparse_correct_kernel<8><<<grid, block, 0, stream>>>(static_cast<const uint16_t*>(W), clean, ent, cnt, keys, P, K, d, V);
  else if (K <= 16)
    sparse_correct_kernel<16><<<grid, block, 0, stream>>>(static_cast<const uint16_t*>(W), clean, ent, cnt, keys, P, K, d, V);
  else
    sparse_correct_kernel<32><<<grid, block, 0, stream>>>(static_cast<const uint16_t*>(W), clean, ent, cnt, keys, P, K, d, V);
  return hipGetLastError();
}

}  // namespace dm
