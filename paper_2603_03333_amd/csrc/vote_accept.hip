// Acceptance step as its own kernel: one workgroup per sequence (see vote_body.hpp).
#include "vote_body.hpp"

namespace dm {
namespace {

__global__ __launch_bounds__(1024) void vote_accept_kernel(const unsigned long long* __restrict__ keys,
                                                          const int32_t* __restrict__ draft_ids,
                                                          const int32_t* __restrict__ parent, int T, int K,
                                                          int Kv, int rule, VoteOut out,
                                                          const float* __restrict__ part_b, JsGeom jg) {
  extern __shared__ int32_t sm[];
  vote_accept_body<false>((int)blockIdx.x, (int)threadIdx.x, (int)blockDim.x, sm, keys, draft_ids, parent, T, K, Kv,
                          rule, out, part_b, jg);
}

}  // namespace

static size_t vote_lds_bytes(int T, int K, int rule) { return vote_lds_ints(T, K, rule) * sizeof(int32_t); }

// Largest scratch any valid call needs: token-level rules T*K <= 16384, T <= 4096 -> 112 KB;
// distribution-level rules T*K <= 8192, T <= 4096 -> 2*T*K + 4*T ints <= 128 KB (T = 4096, K = 2).
static size_t vote_lds_limit() {
  const size_t a = vote_lds_bytes(4096, 4, 0), b = vote_lds_bytes(4096, 2, 2);
  return a > b ? a : b;
}

hipError_t prepare_vote_accept() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&vote_accept_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)vote_lds_limit());
}

hipError_t launch_vote_accept(const unsigned long long* keys, const int32_t* draft_ids, const int32_t* parent,
                              int B, int T, int K, int Kv, int rule, const VoteOut& out, const float* part_b,
                              const JsGeom* jg, hipStream_t stream) {
  if (Kv < 1 || Kv > K) return hipErrorInvalidValue;
  if (rule >= 2 && (part_b == nullptr || jg == nullptr || parent != nullptr || K > kJsMaxK)) return hipErrorInvalidValue;
  if (vote_lds_bytes(T, K, rule) > vote_lds_limit()) return hipErrorInvalidValue;
  const JsGeom geom = jg ? *jg : JsGeom{};
  // the step takes one row per wavefront at a time (a chain of dependent cross-lane steps per row): many rows, many wavefronts
  // (the distribution-level rules also add up T * (K + 1) sums of chunk records, 8 lanes each)
  const unsigned threads = (T > 16 || rule >= 2) ? 1024u : 256u;
  vote_accept_kernel<<<dim3((unsigned)B), dim3(threads), vote_lds_bytes(T, K, rule), stream>>>(keys, draft_ids, parent, T,
                                                                                          K, Kv, rule, out, part_b, geom);
  return hipGetLastError();
}

}  // namespace dm
