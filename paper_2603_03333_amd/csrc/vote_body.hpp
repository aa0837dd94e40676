// Acceptance of draft tokens against the K path tokens of every row: naive token matching
// (Eq. 4), majority (Eq. 7), the JS rule (Eq. 6: the partial sums of the JS kernels are added up
// here, chunks in ascending order) and Algorithm 1 (Eq. 6, else Eq. 7), then the prefix rule of
// speculative decoding (chain) or its extension along parent links (tree).  Written as a device
// function so that it can run as its own kernel (one workgroup per sequence) or as the tail of the
// contraction kernel (by the workgroup that finishes last).
#pragma once
#include "kernels.hpp"

namespace dm {

__host__ __device__ inline size_t vote_lds_ints(int T, int K, int rule) {
  return (size_t)T * K + 3 * (size_t)T + (rule >= 2 ? (size_t)T * (K + 1) : 0);
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(x, off, 64);
    x = o > x ? o : x;
  }
  return x;
}

// The whole acceptance step for sequence b, run by `nthreads` threads (a multiple of 64; thread
// index tid) that may all call __syncthreads().  sm: LDS scratch of vote_lds_ints(T, K, rule) ints.
// COHERENT: the keys were written by other workgroups of the same kernel (argmax merge by atomics),
// so they are read with device-scope atomic loads instead of plain cached loads.
template <bool COHERENT>
__device__ __forceinline__ void vote_accept_body(int b, int tid, int nthreads, int32_t* sm,
                                                 const unsigned long long* keys,
                                                 const int32_t* __restrict__ draft_ids,
                                                 const int32_t* __restrict__ parent, int T, int K, int Kv, int rule,
                                                 const VoteOut& out, const float* __restrict__ part_b,
                                                 const JsGeom& jg) {
  int32_t* ids = sm;            // [T*K] path tokens of this sequence
  int32_t* vid = ids + T * K;   // [T] mode of each row
  int32_t* hitv = vid + T;      // [T] per-row rule result
  int32_t* aux = hitv + T;      // [T] tree: depth of accepted nodes, -1 if rejected
  float* jsv = reinterpret_cast<float*>(aux + T);  // [T][K+1] JS of the K heads, then of the draft (rules 2, 3)

  const int lane = tid & 63, wave = tid >> 6;
  const int nwaves = nthreads >> 6;
  const int TK = T * K;

  // path token = vocabulary index held in the low word of the packed argmax key
  for (int x = tid; x < TK; x += nthreads) {
    const unsigned long long key = COHERENT ? __hip_atomic_load(&keys[(int64_t)b * TK + x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                            : keys[(int64_t)b * TK + x];
    const int32_t id = (int32_t)(0xFFFFFFFFu - (uint32_t)key);
    ids[x] = id;
    if (out.path_ids) out.path_ids[(int64_t)b * TK + x] = id;
  }
  __syncthreads();

  // Eq. (6): total JS of every (row, head) and (row, draft) = its per-chunk partial sums, added by 8
  // lanes per sum: every lane adds every 8th record in ascending order (independent loads, all in
  // flight together), then a butterfly over the 8 lanes - a fixed order, so the result is reproducible
  if (rule >= 2) {
    const int K1 = K + 1;
    const int sub = tid & 7;
    for (int x0 = 0; x0 < T * K1; x0 += nthreads >> 3) {   // uniform trip count: every lane reaches the shuffles
      const int x = x0 + (tid >> 3);
      const bool live = x < T * K1;
      const int t = live ? x / K1 : 0, i = live ? x - t * K1 : 0;
      const bool clean_slot = i >= Kv && i < K;  // slot of the clean path: not a head of the cluster
      double s = 0.0;
      if (live && !clean_slot) {
        const float* src = part_b + (((int64_t)b * T + t) * jg.KS + (i < K ? i : jg.K4)) * jg.NC;
        for (int c = sub; c < jg.NC; c += 8) s += (double)src[c];
      }
#pragma unroll
      for (int off = 4; off >= 1; off >>= 1) s += __shfl_xor(s, off, 8);
      if (!live || sub != 0) continue;
      const float js = clean_slot ? 0.f : (float)s;
      jsv[x] = js;
      if (i < K) {
        if (out.js_heads) out.js_heads[((int64_t)b * T + t) * K + i] = js;
      } else if (out.js_draft) {
        out.js_draft[(int64_t)b * T + t] = draft_ids[(int64_t)b * T + t] >= 0 ? js : -1.0f;
      }
    }
  }

  // mode of the K tokens of each row (ties: smallest id), one wavefront per row
  for (int t = wave; t < T; t += nwaves) {
    const int32_t* row = ids + t * K;
    unsigned long long best = 0;
    for (int i0 = 0; i0 < Kv; i0 += 64) {
      const int i = i0 + lane;
      if (i < Kv) {
        const int32_t mine = row[i];
        uint32_t cnt = 0;
        for (int j = 0; j < Kv; ++j) cnt += (row[j] == mine) ? 1u : 0u;
        const unsigned long long k = ((unsigned long long)cnt << 32) | (0x7FFFFFFFu - (uint32_t)mine);
        best = k > best ? k : best;
      }
    }
    best = wave_max_u64(best);
    if (lane == 0) {
      const int32_t id = (int32_t)(0x7FFFFFFFu - (uint32_t)best);
      vid[t] = id;
      if (out.vote_ids) out.vote_ids[(int64_t)b * T + t] = id;
      if (out.vote_cnt) out.vote_cnt[(int64_t)b * T + t] = (int32_t)(best >> 32);
    }
  }
  __syncthreads();

  // rule result per row (chain: against its own paths; tree: against the parent's paths)
  for (int t = wave; t < T; t += nwaves) {
    int32_t src = t;
    int forced = -1;  // -1: evaluate the rule
    if (parent != nullptr) {
      if (t == 0) {
        forced = 1;
      } else {
        src = parent[(int64_t)b * T + t];
        if (src < 0 || src >= t) forced = 0;
      }
    }
    int h;
    if (forced >= 0) {
      h = forced;
    } else {
      const int32_t g = draft_ids[(int64_t)b * T + t];
      if (rule >= 2) {
        // Eq. (6): JS(phat || pbar) <= max_i JS(p^(i) || pbar), both sides as float; rule 3 = Alg. 1
        const float* row = jsv + t * (K + 1);
        float js_max = -INFINITY;
        for (int i = lane; i < Kv; i += 64) js_max = fmaxf(js_max, row[i]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) js_max = fmaxf(js_max, __shfl_xor(js_max, off, 64));
        const float jd = row[K];
        h = (g >= 0 && jd <= js_max) ? 1 : 0;
        if (rule == 3 && g >= 0 && vid[src] == g) h = 1;
      } else if (g < 0) {
        h = 0;
      } else if (rule == 1) {
        h = (vid[src] == g) ? 1 : 0;
      } else {
        int any = 0;
        for (int i = lane; i < Kv; i += 64) any |= (ids[src * K + i] == g) ? 1 : 0;
        h = __any(any) ? 1 : 0;
      }
    }
    if (lane == 0) {
      hitv[t] = h;
      if (out.hit) out.hit[(int64_t)b * T + t] = (uint8_t)h;
    }
  }
  __syncthreads();

  if (tid == 0) {
    int len, best_node;
    if (parent == nullptr) {
      int n = 0;
      while (n < T && hitv[n]) ++n;
      len = n;
      best_node = n - 1;
      for (int t = 0; t < T; ++t) aux[t] = (t < n) ? 0 : -1;
    } else {
      aux[0] = 0;
      len = 0;
      best_node = 0;
      for (int n = 1; n < T; ++n) {
        const int q = parent[(int64_t)b * T + n];
        int dep = -1;
        if (q >= 0 && q < n && hitv[n] && aux[q] >= 0) dep = aux[q] + 1;
        aux[n] = dep;
        if (dep > len) {
          len = dep;
          best_node = n;
        }
      }
    }
    out.accept_len[b] = len;
    if (out.best_node) out.best_node[b] = best_node;
  }
  __syncthreads();
  if (out.accept_mask)
    for (int t = tid; t < T; t += nthreads) out.accept_mask[(int64_t)b * T + t] = aux[t] >= 0 ? 1 : 0;
}

}  // namespace dm
