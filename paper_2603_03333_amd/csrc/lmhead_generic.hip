// Eq. (3) l = W h^(i) with a fused per-row argmax, on plain fp32 FMA tiles.  Serves the fp32
// storage type and every shape the MFMA kernel does not take; also the second, independent
// GPU implementation the MFMA kernel is compared with in the tests.
//
// Workgroup = 256 threads = 64 masked rows x 64 vocabulary rows, 4 x 4 outputs per thread,
// k in slabs of 16 staged through LDS (stored k-major so the inner loop reads float4), the next
// slab prefetched into registers during the FMAs of the current one.
#include "kernels.hpp"
#include "sampling.hpp"

namespace dm {
namespace {

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }

constexpr int GT = 64;  // tile edge
constexpr int GK = 16;  // k slab

// MODE 0: argmax keys; MODE 1: debug dump of logits[M, dv1 - dv0]; MODE 2: argmax keys and every scaled
// logit stored as [position][vocabulary row][path] for the distribution-level rule.
// SAMPLE (MODE 0 only): arg max over zscale * logit + Gumbel noise = a draw from Softmax(logit / temperature).
template <typename T, int MODE, bool SAMPLE>
__global__ __launch_bounds__(256) void lmhead_generic_kernel(const T* __restrict__ W, const T* __restrict__ A,
                                                             unsigned long long* __restrict__ keys, int64_t M,
                                                             int d, int d_pad, int V, int vtile0,
                                                             float* __restrict__ logits, int dv0, int dv1,
                                                             float scale, LogitStore store, SampleCfg samp) {
  constexpr bool DUMP = MODE == 1;
  __shared__ __attribute__((aligned(16))) float As[GK][GT + 4];
  __shared__ __attribute__((aligned(16))) float Ws[GK][GT + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int64_t m0 = (int64_t)blockIdx.y * GT;
  const int v0 = (vtile0 + (int)blockIdx.x) * GT;

  // loader role: row lr of the tile, 4 consecutive k starting at lk
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  const int64_t arow = m0 + lr;  // always inside the zero-padded workspace
  const int wrow = v0 + lr;

  float acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;

  // slab k0 travels global -> registers while the FMAs of slab k0 - GK run, then registers -> LDS
  float a_reg[4], w_reg[4];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int k = k0 + lk + e;
      a_reg[e] = (k < d_pad) ? to_f32(A[arow * d_pad + k]) : 0.f;
      w_reg[e] = (wrow < V && k < d) ? to_f32(W[(int64_t)wrow * d + k]) : 0.f;
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < d; k0 += GK) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      As[lk + e][lr] = a_reg[e];
      Ws[lk + e][lr] = w_reg[e];
    }
    __syncthreads();
    if (k0 + GK < d) fetch(k0 + GK);
#pragma unroll
    for (int k = 0; k < GK; ++k) {
      const float4 a4 = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      const float4 w4 = *reinterpret_cast<const float4*>(&Ws[k][tx * 4]);
      const float a[4] = {a4.x, a4.y, a4.z, a4.w};
      const float w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
      for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[x][y] = fmaf(a[x], w[y], acc[x][y]);
    }
    __syncthreads();
  }

  if (DUMP) {
    const int nv = dv1 - dv0;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int64_t m = m0 + ty * 4 + x;
      if (m >= M) continue;
      const float sc = (store.clean_last && m % store.K == store.K - 1) ? 1.0f : scale;  // clean path: no 1/(1-p)
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        const int v = v0 + tx * 4 + y;
        if (v >= dv0 && v < dv1 && v < V) logits[m * nv + (v - dv0)] = sc * acc[x][y];
      }
    }
    return;
  }

  if (MODE == 2) {
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int64_t m = m0 + ty * 4 + x;
      if (m >= M) continue;
      const int64_t pos = m / store.K;
      float* row = store.lt + pos * store.V * (int64_t)store.K4 + (m - pos * store.K);
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        const int v = v0 + tx * 4 + y;
        if (v < V) row[(int64_t)v * store.K4] = scale * acc[x][y];
      }
    }
  }

#pragma unroll
  for (int x = 0; x < 4; ++x) {
    float best = -INFINITY;
    uint32_t bv = 0xFFFFFFFFu;
    RowRng rng{0u, 0u, 0u, 0u, false};
    if (SAMPLE) rng = make_row_rng(samp, m0 + ty * 4 + x, M);
    const bool noisy = SAMPLE && rng.on;
    float g[4] = {0.f, 0.f, 0.f, 0.f};
    if (noisy) gumbel4(rng, (uint32_t)(v0 + tx * 4), step_now(samp.step, samp.step_dev), g);
#pragma unroll
    for (int y = 0; y < 4; ++y) {
      const int v = v0 + tx * 4 + y;
      const float val = noisy ? fmaf(acc[x][y], samp.zscale, g[y]) : acc[x][y] + 0.0f;  // -0 -> +0
      if (v < V && (bv == 0xFFFFFFFFu || val > best)) {
        best = val;
        bv = (uint32_t)v;
      }
    }
    unsigned long long key = (bv == 0xFFFFFFFFu) ? 0ull : pack_key(best, bv);
    // the 16 threads that share ty are 16 consecutive lanes of one wavefront
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) {
      const unsigned long long other = __shfl_xor(key, off, 64);
      key = other > key ? other : key;
    }
    const int64_t m = m0 + ty * 4 + x;
    if (tx == 0 && m < M && key != 0ull) atomicMax(&keys[m], key);
  }
}

}  // namespace

hipError_t launch_lmhead_generic(const void* W, const void* a_ws, unsigned long long* keys, const RowGeom& g,
                                 int V, bool is_bf16, float* logits, int v0, int v1, float scale,
                                 const LogitStore& store, const SampleCfg& samp, const LaunchSite& at) {
  const bool dump = logits != nullptr;
  const int tile0 = dump ? v0 / GT : 0;
  const int tile1 = dump ? (v1 + GT - 1) / GT : (V + GT - 1) / GT;
  if (tile1 <= tile0) return hipSuccess;
  const int64_t mtiles = (g.M + GT - 1) / GT;
  if (mtiles > 65535) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(tile1 - tile0), (unsigned)mtiles), block(256);
  const int mode = dump ? 1 : (store.lt != nullptr ? 2 : 0);
#define DM_GEN(T, MODE, SAMPLE)                                                                                   \
  launch_at(lmhead_generic_kernel<T, MODE, SAMPLE>, grid, block, (size_t)0, at, static_cast<const T*>(W),           \
            static_cast<const T*>(a_ws), keys, g.M, g.d, g.d_pad, V, tile0, logits, v0, v1, scale, store, samp)
  const bool sample = mode == 0 && samp.seeds != nullptr;
  if (is_bf16) {
    if (mode == 1) DM_GEN(uint16_t, 1, false); else if (mode == 2) DM_GEN(uint16_t, 2, false);
    else if (sample) DM_GEN(uint16_t, 0, true); else DM_GEN(uint16_t, 0, false);
  } else {
    if (mode == 1) DM_GEN(float, 1, false); else if (mode == 2) DM_GEN(float, 2, false);
    else if (sample) DM_GEN(float, 0, true); else DM_GEN(float, 0, false);
  }
#undef DM_GEN
  return hipGetLastError();
}

}  // namespace dm
