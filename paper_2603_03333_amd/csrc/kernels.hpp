// Launchers of the device kernels behind the C ABI.  All of them only enqueue work on
// `stream`; shapes have been validated by the caller (api.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace dm {

constexpr int kSeedsPerLaunch = 128;  // seeds travel as kernel arguments, this many per launch

struct SeedPack {
  uint64_t s[kSeedsPerLaunch];
};

struct RowGeom {
  int B, T, K, d;
  int64_t M;       // B*T*K real rows
  int64_t M_pad;   // rows of the masked-row workspace (zero rows past M)
  int d_pad;       // columns of the plain workspace layout (zero columns past d)
  uint32_t thr;    // drop threshold floor(p * 2^32)
  uint32_t step;
  const uint32_t* step_dev;  // DEVICE word added to step when the kernels run (nullptr: nothing added)
  int share_pos;   // row word of the counter forced to 0
  int clean_last;  // path K-1 of every row keeps every dimension (the plain LM head)
};

// Counter word 3 of both Philox streams: the step of the call plus, if given, a word the kernels read from
// device memory when they run (so that a captured graph can be replayed with fresh masks and noise).
__device__ __forceinline__ uint32_t step_now(uint32_t step, const uint32_t* step_dev) {
  return step_dev != nullptr ? step + *step_dev : step;
}

// Eq. (1)+(2) without the scale: masked rows a = keep ? h : 0 into the workspace, and the
// per-row argmax keys reset to 0.  layout: plain [M_pad, d_pad], or the order of the B-fragments of the
// MFMA kernels that will read them (16 rows x 32 k).  is_bf16 selects the element type of h and the workspace.
// seeds_dev (optional): DEVICE [B], receives the seeds (for the sampling epilogues of the same call).
// Per-call state of the later kernels of the same call is put back to zero here as well, so that a
// call never depends on an earlier one having run to its end: the election counter of the fused
// acceptance step and the digit histograms of the nucleus search.
struct CallReset {
  unsigned int* counter = nullptr;        // one word, or null
  unsigned long long* zero64 = nullptr;   // n64 words, or null
  int64_t n64 = 0;
};
constexpr int kRowsPlain = 0, kRowsFrag16 = 1;
hipError_t launch_mask_rows(const void* h, void* a_ws, unsigned long long* keys, const uint64_t* seeds_host,
                            const RowGeom& g, bool is_bf16, int layout, uint64_t* seeds_dev,
                            const CallReset& reset, hipStream_t stream);

// Eq. (1) only, bit-packed [M, ceil(d/32)].
hipError_t launch_mask_bits(uint32_t* bits, const uint64_t* seeds_host, const RowGeom& g, hipStream_t stream);

// Where the contraction kernels put every scaled logit when the distribution-level rule needs them
// (Eq. (5), (6)): lt[(pos * V + v) * K4 + i] = logit of path i of position pos at vocabulary row v,
// pos = b * T + t, K4 = K rounded up to a multiple of 4 (16-byte aligned groups; the padding is never
// read as data).  lt == nullptr: nothing is stored.
struct LogitStore {
  float* lt;
  int K, K4, V;
  int clean_last;  // debug dump only: rows of path K-1 are reported without the factor 1/(1-p)
};

// Sampled path tokens (seeds == nullptr: plain arg max).  The contraction epilogues then compare
// zscale * accumulator + Gumbel noise instead of the accumulator (zscale = 1 / ((1-p) tau)).
struct SampleCfg {
  const uint64_t* seeds;  // DEVICE [B], written by the mask kernel of the same call
  float zscale;
  int T, K;
  uint32_t step;
  int clean_last;
  float* noise;
  const uint32_t* step_dev = nullptr;  // as in RowGeom  // DEVICE scratch, 256 KB per workgroup of the 256 x 256 kernel (its copy wavefronts draw the noise), or null
};

// Where a contraction kernel is launched: the stream and, optionally, two events that receive the
// begin and end timestamps of that launch itself.  Events recorded on the stream before and after
// a launch also span the dispatch gap in front of the kernel (measured: 5-9 us on a 160 us kernel).
struct LaunchSite {
  hipStream_t stream;
  hipEvent_t start = nullptr, stop = nullptr;
};

template <typename... KArgs, typename... Args>
inline void launch_at(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, const LaunchSite& at,
                      Args... args) {
  if (at.start != nullptr)
    hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, at.stream, at.start, at.stop, 0, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds_bytes, at.stream, args...);
}

// Eq. (3) + per-row argmax, generic fp32-FMA tiles.  a_ws plain layout.  If logits != null the
// kernel instead stores scale * accumulator for v in [v0, v1) and touches no keys.
hipError_t launch_lmhead_generic(const void* W, const void* a_ws, unsigned long long* keys, const RowGeom& g,
                                 int V, bool is_bf16, float* logits, int v0, int v1, float scale,
                                 const LogitStore& store, const SampleCfg& samp, const LaunchSite& at);

// Eq. (3) + per-row argmax on bf16 MFMA; a_ws in fragment order (kRowsFrag16); d % 64 == 0.
struct VoteFuse;
// fuse (optional): also run the acceptance step in the same launch (token-level rules, no dump, no store).
// *fused is set when that was done.
hipError_t launch_lmhead_mfma(const void* W, const void* a_ws, unsigned long long* keys, const RowGeom& g,
                              int V, int num_cu, float* logits, int v0, int v1, float scale,
                              const LogitStore& store, const SampleCfg& samp, const VoteFuse* fuse, bool* fused,
                              const LaunchSite& at);
hipError_t prepare_lmhead_mfma();  // raises the dynamic-LDS limit of the kernels once per process

// Same contract for more than 128 masked rows (256 x 256 tiles); needs M_pad % 256 == 0.
hipError_t launch_lmhead_mfma_big(const void* W, const void* a_ws, unsigned long long* keys, const RowGeom& g,
                                  int V, int num_cu, float* logits, int v0, int v1, float scale,
                                  const LogitStore& store, const SampleCfg& samp, const LaunchSite& at);
hipError_t prepare_lmhead_mfma_big();

// Distribution-level rule (Eq. (5), (6)) over the stored logits, in two passes over the vocabulary;
// each workgroup takes kJsChunk vocabulary rows of one position and leaves partial sums that the
// next kernel adds up in a fixed order (so results do not depend on scheduling).
constexpr int kJsChunk = 4096;  // vocabulary rows per workgroup (1024 threads)
constexpr int kJsMaxK = 64;     // paths per row the distribution-level rule takes
struct JsGeom {
  int P;    // positions B*T
  int K, K4;  // rows per position in the logit store (K4 = K rounded up to a multiple of 4)
  int KU;     // heads the rule uses: K, or K - 1 when the last path is the clean one
  int V;
  int NC;   // ceil(V / kJsChunk)
  int KS;   // slots per position in part_a / part_b (layout [pos][slot][chunk]): K4 + 4
};
// Pass 1: part_a[pos][i][c] = sum over chunk c of exp(l_i[v] - max_v l_i) for path i < K;
// slots K4 / K4+1 = (max, sum of exp relative to it) of the mean logits over the chunk.
hipError_t launch_js_stats(const float* lt, const unsigned long long* keys, float* part_a, const JsGeom& g,
                           float scale, hipStream_t stream);
// Pass 2: part_b[pos][i][c] = chunk's share of JS(p^(i) || pbar) for i < K; slot K4 = of JS(phat || pbar).
hipError_t launch_js_terms(const float* lt, const unsigned long long* keys, const float* part_a,
                           const float* draft_probs, const int32_t* draft_ids, float* part_b, const JsGeom& g,
                           float scale, hipStream_t stream);

// Eq. (4)/(7), Eq. (6), Alg. 1, prefix / tree rule.  One workgroup per sequence.
struct VoteOut {
  int32_t* accept_len;
  int32_t* best_node;
  uint8_t* accept_mask;
  uint8_t* hit;
  int32_t* path_ids;
  int32_t* vote_ids;
  int32_t* vote_cnt;
  float* js_draft;  // [B,T]   (distribution-level rules only)
  float* js_heads;  // [B,T,K]
};
// part_b / jg: partial JS sums of launch_js_terms (rules 2 and 3), else nullptr.
// Acceptance step run as the tail of the contraction kernel: every workgroup bumps `counter` when
// its argmax keys are merged, and the workgroup that finds it at (workgroups - 1) runs the step for
// all B sequences.  The mask kernel of every call puts the counter to 0.  counter == nullptr: not fused.
struct VoteFuse {
  unsigned int* counter;
  const int32_t* draft_ids;
  const int32_t* parent;
  int B, T, K, Kv, rule;
  VoteOut out;
};

// Kv: paths the rules and the vote use (K, or K - 1 with a clean last path).
hipError_t launch_vote_accept(const unsigned long long* keys, const int32_t* draft_ids, const int32_t* parent,
                              int B, int T, int K, int Kv, int rule, const VoteOut& out, const float* part_b,
                              const JsGeom* jg, hipStream_t stream);
hipError_t prepare_vote_accept();

// The path logits as clean row minus per-path corrections over the dropped dimensions (sparse_correction.hip).
// ent: [rows][d / 64][64] words (dimension inside the slab | bf16 bits of h << 16), cnt: [rows][d / 64];
// clean: [positions][V] logits of the undropped rows.  bf16, d % 64 == 0, K <= kSparseMaxK.
constexpr int kSparseMaxK = 32;
hipError_t launch_drop_lists(const void* h, uint32_t* ent, uint32_t* cnt, unsigned long long* keys,
                             const uint64_t* seeds_host, const RowGeom& g, hipStream_t stream);
hipError_t launch_sparse_correct(const void* W, const float* clean, const uint32_t* ent, const uint32_t* cnt,
                                 unsigned long long* keys, int P, int K, int d, int V, hipStream_t stream);

// Measurement aid: plain streaming read of `bytes` bytes (a multiple of 16) at src; sink: one device word.
hipError_t launch_stream_read(const void* src, size_t bytes, int num_cu, unsigned int* sink, hipStream_t stream);

// Packed argmax key: larger logit wins, then smaller vocabulary index.  Key 0 = "nothing yet".
__host__ __device__ inline unsigned long long pack_key(float val, uint32_t v) {
  union { float f; uint32_t u; } c;
  c.f = val;
  uint32_t u = c.u;
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((unsigned long long)u << 32) | (unsigned long long)(0xFFFFFFFFu - v);
}

// Sampled path tokens restricted to the nucleus (top-p set) of Softmax(l / tau), over the stored logits:
// a histogram + scan pass finds the leading digit of each row's threshold, the draw pass draws below it and
// lists the tokens of that digit, a last pass settles the threshold and the draw on the list.
constexpr int kNucChunk = 1024;  // vocabulary rows per workgroup
constexpr int kNucMaxK = 64;     // paths per row
struct NucGeom {
  int P;    // positions B*T
  int K;    // rows per position in the key arrays
  int K4;   // floats per (position, vocabulary row) in the store
  int KP;   // K4 rounded up to a power of two (thread mapping)
  int KU;   // paths that draw (K, or K-1 when the last path is the clean one)
  int V;
  int cap;  // entries per row of the candidate lists
  int fine; // the first histogram has fine bins next to the row's maximum (see nucleus_fine_bins)
};
constexpr int kNucFineMaxKP = 32;
// Whether a call uses the fine bins.  They cost the histogram and draw passes 7 % (more instructions per
// element, more non-empty bins to add to memory) and matter for rows so flat that an eighth of the
// vocabulary lies within 0.125 * temperature of the threshold in logit units: taken from a temperature of 2
// on, where synthetic Gaussian rows start to come close to that; they double the LDS of the histogram pass, so
// only up to 32 paths.
inline bool nucleus_fine_bins(int KP, float temperature) { return KP <= kNucFineMaxKP && temperature >= 2.0f; }
struct NucBuffers {
  unsigned long long* hist;    // [rows][512] masses per leading digit, 256 coarse bins then 256 fine ones; zeroed by the
                               // mask kernel of the call, and by the scan
  uint32_t* digit0;            // [rows] leading digit of the threshold | (its position in the key, 16 or 12) << 16
  unsigned long long* below;   // [rows] mass of the elements below that digit
  unsigned long long* target;  // [rows] mass the nucleus has to reach
  unsigned long long* keys_s;  // [rows] packed keys of the drawn tokens
  uint2* cand;                 // [rows][cap] (logit bits, token) of the tokens that share the threshold's leading digit
  uint32_t* cand_n;            // [rows] how many there are (beyond cap: the list did not fit)
};
// Entries per row that the lists get for a vocabulary of V tokens: an eighth of it (a flat Gaussian row puts a
// few per cent of its tokens on the list), at least 1024.
inline int64_t nucleus_list_capacity(int64_t V) { return V / 8 > 1024 ? V / 8 : 1024; }
hipError_t launch_nucleus(const float* lt, const unsigned long long* keys, const NucBuffers& nb, const NucGeom& g,
                          const SampleCfg& samp, float scale, float inv_tau, double top_p, hipStream_t stream);
hipError_t prepare_nucleus();


}  // namespace dm
