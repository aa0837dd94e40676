// Keep-masks of Eq. (1) and masked rows of Eq. (2) (scale deferred: it cannot change an argmax).
//
// mask_rows_kernel: one thread per (row, group of 8 dimensions).  Rows are the fastest index
// across a wavefront, so the K paths of one position read the same 16 bytes of h (a broadcast
// in the memory pipeline) and 32 consecutive rows write 512 contiguous bytes of the workspace.
// Two Philox calls give the 8 keep bits.  The thread that handles dimension group 0 also
// resets the row's packed argmax key; the first launch of a call also puts the per-call state of
// the later kernels (CallReset) back to zero.
#include "kernels.hpp"
#include "philox.hpp"

namespace dm {

namespace {

template <typename T>
struct Vec8;
template <>
struct __attribute__((aligned(16))) Vec8<float> {
  float v[8];
};
template <>
struct __attribute__((aligned(16))) Vec8<uint16_t> {
  uint16_t v[8];
};

// T = float or uint16_t (bfloat16 bit pattern; selecting between a value and +0 needs no arithmetic)
template <typename T, int LAYOUT>
__global__ __launch_bounds__(256) void mask_rows_kernel(const T* __restrict__ h, T* __restrict__ a_ws,
                                                        unsigned long long* __restrict__ keys, SeedPack seeds,
                                                        RowGeom g, int64_t row0, int64_t nrows, int b0,
                                                        uint64_t* __restrict__ seeds_dev, int nb,
                                                        CallReset reset) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (seeds_dev != nullptr && idx < nb) seeds_dev[b0 + idx] = seeds.s[idx];  // for the sampling epilogues
  if (reset.counter != nullptr && idx == 0) *reset.counter = 0u;
  for (int64_t x = idx; x < reset.n64; x += (int64_t)gridDim.x * blockDim.x) reset.zero64[x] = 0ull;
  const int ngroups = g.d_pad >> 3;
  if (idx >= nrows * ngroups) return;
  const int64_t r = row0 + idx % nrows;
  const uint32_t o = (uint32_t)(idx / nrows);

  Vec8<T> out;
#pragma unroll
  for (int e = 0; e < 8; ++e) out.v[e] = T(0);

  if (r < g.M && (int)(8u * o) < g.d) {
    const int TK = g.T * g.K;
    const int b = (int)(r / TK);
    const int rem = (int)(r - (int64_t)b * TK);
    const int t = rem / g.K;
    const int i = rem - t * g.K;
    const uint64_t seed = seeds.s[b - b0];
    const uint32_t bits = (g.clean_last && i == g.K - 1)
                              ? 0xFFu
                              : keep_bits8(o, g.share_pos ? 0u : (uint32_t)t, (uint32_t)i, step_now(g.step, g.step_dev),
                                           (uint32_t)seed, (uint32_t)(seed >> 32), g.thr);
    const T* src = h + ((int64_t)b * g.T + t) * g.d + 8 * (int64_t)o;
    if ((g.d & 7) == 0) {
      const Vec8<T> in = *reinterpret_cast<const Vec8<T>*>(src);
#pragma unroll
      for (int e = 0; e < 8; ++e) out.v[e] = ((bits >> e) & 1u) ? in.v[e] : T(0);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if ((int)(8u * o) + e < g.d) out.v[e] = ((bits >> e) & 1u) ? src[e] : T(0);
    }
  }

  int64_t dst;
  if (LAYOUT == kRowsFrag16) {
    // B-operand fragments of v_mfma_f32_16x16x32_bf16: fragment (k-step ks of 32, row tile mt of 16) is
    // 64 lanes x 8 elements; lane = (row % 16) + 16 * ((k % 32) / 8), element = k % 8.
    const int64_t mt_total = g.M_pad >> 4;
    dst = ((((int64_t)(o >> 2) * mt_total + (r >> 4)) * 64) + (r & 15) + 16 * (o & 3)) * 8;
  } else {
    dst = r * g.d_pad + 8 * (int64_t)o;
  }
  *reinterpret_cast<Vec8<T>*>(a_ws + dst) = out;
  if (o == 0 && keys != nullptr) keys[r] = 0ull;
}

__global__ __launch_bounds__(256) void mask_bits_kernel(uint32_t* __restrict__ bits, SeedPack seeds, RowGeom g,
                                                        int64_t row0, int64_t nrows, int b0) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nwords = (g.d + 31) >> 5;
  if (idx >= nrows * nwords) return;
  const int64_t r = row0 + idx / nwords;
  const uint32_t w = (uint32_t)(idx % nwords);
  const int TK = g.T * g.K;
  const int b = (int)(r / TK);
  const int rem = (int)(r - (int64_t)b * TK);
  const int t = rem / g.K;
  const int i = rem - t * g.K;
  const uint64_t seed = seeds.s[b - b0];
  uint32_t word = 0;
  if (g.clean_last && i == g.K - 1) {
    word = 0xFFFFFFFFu;
  } else {
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q)
      word |= keep_bits8(4u * w + q, g.share_pos ? 0u : (uint32_t)t, (uint32_t)i, step_now(g.step, g.step_dev), (uint32_t)seed,
                         (uint32_t)(seed >> 32), g.thr)
              << (8u * q);
  }
  const int valid = g.d - 32 * (int)w;  // dimensions of this word that exist
  if (valid < 32) word &= (1u << valid) - 1u;
  bits[r * nwords + w] = word;
}

template <typename T, int SW>
hipError_t run_mask_rows(const void* h, void* a_ws, unsigned long long* keys, const uint64_t* seeds_host,
                         const RowGeom& g, uint64_t* seeds_dev, const CallReset& reset, hipStream_t stream) {
  const int64_t TK = (int64_t)g.T * g.K;
  for (int b0 = 0; b0 < g.B; b0 += kSeedsPerLaunch) {
    const int nb = (g.B - b0 < kSeedsPerLaunch) ? (g.B - b0) : kSeedsPerLaunch;
    SeedPack sp;
    for (int q = 0; q < kSeedsPerLaunch; ++q) sp.s[q] = (q < nb) ? seeds_host[b0 + q] : 0ull;
    const int64_t row0 = (int64_t)b0 * TK;
    // the last launch also zero-fills the padding rows M .. M_pad
    const int64_t row1 = (b0 + nb == g.B) ? g.M_pad : (int64_t)(b0 + nb) * TK;
    const int64_t nrows = row1 - row0;
    const int64_t nthreads = nrows * (g.d_pad >> 3);
    const int64_t nblocks = (nthreads + 255) / 256;
    if (nblocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    mask_rows_kernel<T, SW><<<dim3((unsigned)nblocks), dim3(256), 0, stream>>>(
        static_cast<const T*>(h), static_cast<T*>(a_ws), keys, sp, g, row0, nrows, b0, seeds_dev, nb,
        b0 == 0 ? reset : CallReset{});
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

hipError_t launch_mask_rows(const void* h, void* a_ws, unsigned long long* keys, const uint64_t* seeds_host,
                            const RowGeom& g, bool is_bf16, int layout, uint64_t* seeds_dev,
                            const CallReset& reset, hipStream_t stream) {
  if (is_bf16) {
    switch (layout) {
      case kRowsPlain: return run_mask_rows<uint16_t, kRowsPlain>(h, a_ws, keys, seeds_host, g, seeds_dev, reset, stream);
      case kRowsFrag16:
        if (g.d_pad % 32 != 0 || g.M_pad % 16 != 0) return hipErrorInvalidValue;
        return run_mask_rows<uint16_t, kRowsFrag16>(h, a_ws, keys, seeds_host, g, seeds_dev, reset, stream);
      default: return hipErrorInvalidValue;
    }
  }
  if (layout != kRowsPlain) return hipErrorInvalidValue;
  return run_mask_rows<float, kRowsPlain>(h, a_ws, keys, seeds_host, g, seeds_dev, reset, stream);
}

hipError_t launch_mask_bits(uint32_t* bits, const uint64_t* seeds_host, const RowGeom& g, hipStream_t stream) {
  const int64_t TK = (int64_t)g.T * g.K;
  const int nwords = (g.d + 31) >> 5;
  for (int b0 = 0; b0 < g.B; b0 += kSeedsPerLaunch) {
    const int nb = (g.B - b0 < kSeedsPerLaunch) ? (g.B - b0) : kSeedsPerLaunch;
    SeedPack sp;
    for (int q = 0; q < kSeedsPerLaunch; ++q) sp.s[q] = (q < nb) ? seeds_host[b0 + q] : 0ull;
    const int64_t row0 = (int64_t)b0 * TK;
    const int64_t nrows = (int64_t)nb * TK;
    const int64_t nblocks = (nrows * nwords + 255) / 256;
    if (nblocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    mask_bits_kernel<<<dim3((unsigned)nblocks), dim3(256), 0, stream>>>(bits, sp, g, row0, nrows, b0);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace dm
