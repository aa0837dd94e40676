// C ABI of the DropMatch verify step (see include/dropmatch.h for the contract).
#include "../../include/dropmatch.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "kernels.hpp"

struct dm_ctx {
  int device = 0;
  int num_cu = 0;
  int64_t max_rows = 0;
  int32_t max_d = 0, max_V = 0;
  int64_t rows_pad = 0;  // max_rows rounded up to 256
  int32_t d_pad = 0;     // max_d rounded up to 64
  void* a_ws = nullptr;               // masked rows
  unsigned long long* keys = nullptr; // packed (logit, index) argmax per row
  unsigned int* done = nullptr;       // workgroups done, for the acceptance step fused into the contraction
  uint64_t* seeds_dev = nullptr;      // seeds of the current call, for the sampling epilogues
  float* noise = nullptr;             // Gumbel noise of one tile per workgroup of the 256 x 256 kernel (allocated on first use)
  // sparse-correction option: clean logits [positions][V], dropped-dimension lists (allocated on first use)
  float* sp_clean = nullptr;
  size_t sp_clean_floats = 0;
  uint32_t* sp_ent = nullptr;
  uint32_t* sp_cnt = nullptr;
  size_t sp_ent_words = 0, sp_cnt_words = 0;
  bool borrowed = false;              // the workspace is the static device array: nothing is allocated or freed
  // distribution-level rule (dm_reserve_js): stored logits and per-chunk partial sums
  float* lt = nullptr;
  size_t lt_floats = 0;
  float* part_a = nullptr;
  float* part_b = nullptr;
  size_t part_floats = 0;
  // nucleus sampling (also dm_reserve_js): per-row digit histograms, search state, keys of the drawn tokens
  dm::NucBuffers nuc{};
  int64_t nuc_cap = 0;
  size_t nuc_rows = 0;
  char err[512] = {0};
  // measurement aid: kEv events per recorded call
  hipEvent_t* ev = nullptr;
  int prof_enabled = 0;
  int prof_calls = 0;
  // per recorded call: bit 0 = stage 2 ran (JS pass 1, or all nucleus passes), bit 1 = separate vote kernel, bit 2 = JS pass 2
  uint8_t prof_kind[DM_PROFILE_MAX_CALLS] = {};
  int prof_stride = 1;  // events are recorded on every prof_stride-th verify call
  int prof_seen = 0;    // verify calls since profiling was switched on
};

namespace {

constexpr int kEv = 6;  // events per recorded call: before mask | lmhead | js_stats | js_terms | vote | end

thread_local char g_err[512] = {0};  // failures that have no context (dm_create, NULL ctx), per host thread

dm_status fail(dm_ctx* ctx, dm_status st, const char* fmt, ...) {
  char* buf = ctx ? ctx->err : g_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, 512, fmt, ap);
  va_end(ap);
  return st;
}

dm_status fail_hip(dm_ctx* ctx, const char* what, hipError_t e) {
  return fail(ctx, DM_EHIP, "%s: %s", what, hipGetErrorString(e));
}

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
    if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
  }
  ~DeviceGuard() {
    int cur = -1;
    if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

// ------------------------------------------------------------------ workspace for callers that cannot allocate
// One array per GPU, held by every device the library's code object is loaded on until the process
// ends.  In host code `dm_static_scratch` is only a handle for hipGetSymbolAddress: the device address
// it returns (per device) is what kernels, copies and fills get.
constexpr size_t kStaticRowBytes = (size_t)DM_STATIC_MAX_WS_BYTES;         // masked rows
constexpr size_t kStaticKeysOff = kStaticRowBytes;                         // DM_STATIC_MAX_ROWS packed keys
constexpr size_t kStaticSeedsOff = kStaticKeysOff + (size_t)DM_STATIC_MAX_ROWS * 8;  // as many seeds
constexpr size_t kStaticDoneOff = kStaticSeedsOff + (size_t)DM_STATIC_MAX_ROWS * 8;  // election counter
constexpr size_t kStaticBytes = kStaticDoneOff + 256;
static_assert(kStaticRowBytes % 256 == 0 && DM_STATIC_MAX_ROWS % 256 == 0, "every part starts 256-byte aligned");
static __device__ __align__(256) unsigned char dm_static_scratch[kStaticBytes];

constexpr int kMaxStaticDevices = 64;
struct StaticSlot {
  bool ready = false;
  dm_ctx ctx;  // a context whose workspace pointers point into the device's copy of the array
};
StaticSlot g_static[kMaxStaticDevices];
std::mutex g_static_mutex;

// Set-up of device `device`, once: address of its copy of the array, device properties, LDS limits of
// the kernels.  No allocation.  On failure the message is left for dm_last_error(NULL).
dm_status static_context(int device, dm_ctx** out) {
  *out = nullptr;
  if (device < 0 || device >= kMaxStaticDevices)
    return fail(nullptr, DM_EINVAL, "device %d not in 0..%d", device, kMaxStaticDevices - 1);
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticSlot& slot = g_static[device];
  if (slot.ready) {
    *out = &slot.ctx;
    return DM_OK;
  }
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess) return fail_hip(nullptr, "hipGetDeviceCount", e);
  if (device >= ndev) return fail(nullptr, DM_EINVAL, "device %d not in 0..%d", device, ndev - 1);
  DeviceGuard guard(device);
  if (!guard.ok) return fail(nullptr, DM_EHIP, "cannot select device %d", device);
  hipDeviceProp_t prop;
  if ((e = hipGetDeviceProperties(&prop, device)) != hipSuccess) return fail_hip(nullptr, "hipGetDeviceProperties", e);
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return fail(nullptr, DM_EUNSUPPORTED, "device %d is %s; this library is built for gfx950 only", device, prop.gcnArchName);
  // the device's own copy of the array (the device is current here)
  unsigned char* base = nullptr;
  if ((e = hipGetSymbolAddress((void**)&base, HIP_SYMBOL(dm_static_scratch))) != hipSuccess)
    return fail_hip(nullptr, "hipGetSymbolAddress(static workspace)", e);
  if (base == nullptr) return fail(nullptr, DM_EHIP, "hipGetSymbolAddress(static workspace) returned no address");
  if ((e = dm::prepare_lmhead_mfma()) != hipSuccess || (e = dm::prepare_lmhead_mfma_big()) != hipSuccess ||
      (e = dm::prepare_vote_accept()) != hipSuccess)
    return fail_hip(nullptr, "raising the dynamic LDS limit", e);
  dm_ctx& c = slot.ctx;
  c.device = device;
  c.num_cu = prop.multiProcessorCount;
  c.max_rows = DM_STATIC_MAX_ROWS;
  c.max_d = 0x7FFFFFFF;  // bounded by the byte size of the masked rows instead
  c.max_V = 0x7FFFFFFF;
  c.rows_pad = DM_STATIC_MAX_ROWS;
  c.a_ws = base;
  c.keys = reinterpret_cast<unsigned long long*>(base + kStaticKeysOff);
  c.seeds_dev = reinterpret_cast<uint64_t*>(base + kStaticSeedsOff);
  c.done = reinterpret_cast<unsigned int*>(base + kStaticDoneOff);
  c.borrowed = true;
  slot.ready = true;
  *out = &c;
  return DM_OK;
}

// Reason a parameter block is unusable, or nullptr.
const char* check_params(const dm_params* p, char* scratch, size_t n) {
  if (!p) return "params is NULL";
  if (p->B < 1) return "B must be >= 1";
  if (p->T < 1 || p->T > DM_MAX_ROWS_PER_SEQ) {
    snprintf(scratch, n, "T must be in 1..%d", DM_MAX_ROWS_PER_SEQ);
    return scratch;
  }
  if (p->K < 1 || p->K > DM_MAX_K) {
    snprintf(scratch, n, "K must be in 1..%d", DM_MAX_K);
    return scratch;
  }
  if ((int64_t)p->T * p->K > DM_MAX_TK) {
    snprintf(scratch, n, "T*K must be <= %d", DM_MAX_TK);
    return scratch;
  }
  if (p->d < 1) return "d must be >= 1";
  if (p->V < 1) return "V must be >= 1";
  if ((int64_t)p->B * p->T * p->K > (int64_t)1 << 40) return "B*T*K too large";
  if (p->dtype != DM_F32 && p->dtype != DM_BF16) return "dtype must be DM_F32 or DM_BF16";
  if (!(p->p >= 0.0f && p->p < 1.0f)) return "p must satisfy 0 <= p < 1";
  if (p->rule < DM_RULE_ANY || p->rule > DM_RULE_JS_OR_MAJORITY) return "rule must be one of the DM_RULE_* values";
  if (p->rule >= DM_RULE_JS && p->K > DM_MAX_K_JS) {
    snprintf(scratch, n, "the distribution-level rules take K <= %d", DM_MAX_K_JS);
    return scratch;
  }
  if (p->rule >= DM_RULE_JS && (int64_t)p->T * p->K > DM_MAX_TK_JS) {
    snprintf(scratch, n, "the distribution-level rules take T*K <= %d", DM_MAX_TK_JS);
    return scratch;
  }
  if (p->rule >= DM_RULE_JS && p->parent != nullptr)
    return "the distribution-level rules are defined for chains only (parent must be NULL)";
  if (p->flags & ~(DM_FLAG_SHARE_MASK_ACROSS_POS | DM_FLAG_FORCE_GENERIC | DM_FLAG_CLEAN_LAST_PATH | DM_FLAG_SEPARATE_VOTE |
                   DM_FLAG_SAMPLE_PATHS | DM_FLAG_SPARSE_CORRECTION))
    return "unknown bits in flags";
  if ((p->flags & DM_FLAG_CLEAN_LAST_PATH) && p->K < 2) return "DM_FLAG_CLEAN_LAST_PATH needs K >= 2";
  if (p->flags & DM_FLAG_SAMPLE_PATHS) {
    if (!(p->temperature > 0.0f) || !std::isfinite(p->temperature))
      return "DM_FLAG_SAMPLE_PATHS needs a finite temperature > 0";
    if (p->rule >= DM_RULE_JS) return "sampled path tokens go with the token-level rules only";
    if (!(p->top_p >= 0.0f && p->top_p <= 1.0f)) return "top_p must satisfy 0 <= top_p <= 1 (0 and 1: no truncation)";
    if (p->top_p > 0.0f && p->top_p < 1.0f) {
      if (p->K > DM_MAX_K_JS) {
        snprintf(scratch, n, "nucleus sampling takes K <= %d", DM_MAX_K_JS);
        return scratch;
      }
      if ((int64_t)p->T * p->K > DM_MAX_TK_JS) {
        snprintf(scratch, n, "nucleus sampling takes T*K <= %d", DM_MAX_TK_JS);
        return scratch;
      }
    }
  }
  if (!p->seeds) return "seeds is NULL";
  return nullptr;
}

bool use_mfma(const dm_params* p) {
  return p->dtype == DM_BF16 && (p->d % 64) == 0 && !(p->flags & DM_FLAG_FORCE_GENERIC);
}

int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Geometry of a call inside the limits of the context, or an error.
dm_status make_geom(dm_ctx* ctx, const dm_params* p, bool mfma, dm::RowGeom* g) {
  char scratch[128];
  if (const char* why = check_params(p, scratch, sizeof scratch)) return fail(ctx, DM_EINVAL, "%s", why);
  const int64_t M = (int64_t)p->B * p->T * p->K;
  if (M > ctx->max_rows) return fail(ctx, DM_EINVAL, "B*T*K = %lld exceeds the context's max_rows %lld", (long long)M, (long long)ctx->max_rows);
  if (p->d > ctx->max_d) return fail(ctx, DM_EINVAL, "d = %d exceeds the context's max_d %d", p->d, ctx->max_d);
  if (p->V > ctx->max_V) return fail(ctx, DM_EINVAL, "V = %d exceeds the context's max_V %d", p->V, ctx->max_V);
  g->B = p->B;
  g->T = p->T;
  g->K = p->K;
  g->d = p->d;
  g->M = M;
  // MFMA kernels: up to 128 rows in 32-row tiles, beyond that in 256-row tiles
  g->M_pad = mfma ? (M <= 128 ? round_up(M, 32) : round_up(M, 256)) : round_up(M, 128);
  g->d_pad = (int)round_up(p->d, 64);
  g->thr = (uint32_t)std::floor((double)p->p * 4294967296.0);
  g->step = p->step;
  g->step_dev = p->step_dev;
  g->share_pos = (p->flags & DM_FLAG_SHARE_MASK_ACROSS_POS) ? 1 : 0;
  g->clean_last = (p->flags & DM_FLAG_CLEAN_LAST_PATH) ? 1 : 0;
  return DM_OK;
}


// Eq. (1)-(3) + argmax keys; shared by dropmatch_verify and dm_debug_logits.
// `ev` (optional): 3 events recorded before the mask kernel, between the two kernels, after.
dm_status run_contraction(dm_ctx* ctx, const dm_params* p, const dm::RowGeom& g, bool mfma, const void* h,
                          const void* W, float* logits, int v0, int v1, hipStream_t s, hipEvent_t* ev = nullptr,
                          dm::LogitStore store = dm::LogitStore{nullptr, 0, 0, 0, 0},
                          const dm::VoteFuse* fuse = nullptr, bool* fused = nullptr, int64_t nucleus_rows = 0) {
  if (fused) *fused = false;
  store.K = p->K;  // the debug dump needs K and the clean-path flag even when nothing is stored
  store.clean_last = g.clean_last;
  const bool bf16 = p->dtype == DM_BF16;
  const bool all_stages = ctx->prof_enabled == 1;  // 2: only the contraction kernel is bracketed
  if (ev && all_stages) (void)hipEventRecord(ev[0], s);
  const bool want_seeds = (p->flags & DM_FLAG_SAMPLE_PATHS) && logits == nullptr;
  const bool sample = want_seeds && store.lt == nullptr;  // stored logits: the draw is made from them afterwards
  // the first kernel of the call also puts back to zero what the later ones count in
  dm::CallReset reset;
  reset.counter = ctx->done;
  if (nucleus_rows > 0) {
    reset.zero64 = ctx->nuc.hist;
    reset.n64 = nucleus_rows * 512;
  }
  const int row_layout = mfma ? dm::kRowsFrag16 : dm::kRowsPlain;
  hipError_t e = dm::launch_mask_rows(h, ctx->a_ws, ctx->keys, p->seeds, g, bf16, row_layout,
                                      want_seeds ? ctx->seeds_dev : nullptr, reset, s);
  if (e != hipSuccess) return fail_hip(ctx, "mask_rows launch", e);
  // all stages: events on the stream around every kernel; otherwise the two events take the
  // timestamps of the contraction launch itself
  dm::LaunchSite at{s};
  if (ev && all_stages) (void)hipEventRecord(ev[1], s);
  if (ev && !all_stages) {
    at.start = ev[1];
    at.stop = ev[2];
  }
  const float scale = (float)(1.0 / (1.0 - (double)p->p));
  dm::SampleCfg samp{nullptr, 0.f, p->T, p->K, p->step, g.clean_last, ctx->noise, p->step_dev};
  if (sample) {
    samp.seeds = ctx->seeds_dev;
    samp.zscale = (float)(1.0 / (1.0 - (double)p->p) / (double)p->temperature);
  }
  if (mfma && g.M <= 128)
    e = dm::launch_lmhead_mfma(W, ctx->a_ws, ctx->keys, g, p->V, ctx->num_cu, logits, v0, v1, scale, store, samp, fuse, fused, at);
  else if (mfma)
    e = dm::launch_lmhead_mfma_big(W, ctx->a_ws, ctx->keys, g, p->V, ctx->num_cu, logits, v0, v1, scale, store, samp, at);
  else
    e = dm::launch_lmhead_generic(W, ctx->a_ws, ctx->keys, g, p->V, bf16, logits, v0, v1, scale, store, samp, at);
  if (e != hipSuccess) return fail_hip(ctx, "lmhead launch", e);
  if (ev && all_stages) (void)hipEventRecord(ev[2], s);
  return DM_OK;
}

void free_nucleus(dm_ctx* ctx) {
  void* const bufs[] = {ctx->nuc.hist, ctx->nuc.digit0, ctx->nuc.below, ctx->nuc.target,
                        ctx->nuc.keys_s, ctx->nuc.cand, ctx->nuc.cand_n};
  for (void* b : bufs)
    if (b) (void)hipFree(b);
  ctx->nuc = dm::NucBuffers{};
  ctx->nuc_rows = 0;
  ctx->nuc_cap = 0;
}

void drop_events(dm_ctx* ctx) {
  if (!ctx->ev) return;
  for (int i = 0; i < kEv * DM_PROFILE_MAX_CALLS; ++i)
    if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
  delete[] ctx->ev;
  ctx->ev = nullptr;
}

// Path tokens by "clean row minus corrections over the dropped dimensions" (sparse_correction.hip):
// the clean logits of the B*T positions from the contraction kernel (one undropped row per position,
// all logits kept), the dropped-dimension lists, then the corrections and the arg max.
dm_status run_sparse_correction(dm_ctx* ctx, const dm_params* prm, const dm::RowGeom& g, const void* h, const void* W,
                                hipStream_t s) {
  const int64_t P = (int64_t)prm->B * prm->T;
  if (P > 0x7FFFFFFF) return fail(ctx, DM_EINVAL, "B*T too large");
  const size_t clean_floats = (size_t)P * (size_t)prm->V;
  const size_t nslab = (size_t)prm->d / 64;
  const size_t ent_words = (size_t)g.M * nslab * 64, cnt_words = (size_t)g.M * nslab;
  if (clean_floats > ctx->sp_clean_floats || ent_words > ctx->sp_ent_words || cnt_words > ctx->sp_cnt_words) {
    if (hipDeviceSynchronize() != hipSuccess) return fail(ctx, DM_EHIP, "device synchronisation failed before reallocating");
    if (ctx->sp_clean) (void)hipFree(ctx->sp_clean);
    if (ctx->sp_ent) (void)hipFree(ctx->sp_ent);
    if (ctx->sp_cnt) (void)hipFree(ctx->sp_cnt);
    ctx->sp_clean = nullptr;
    ctx->sp_ent = ctx->sp_cnt = nullptr;
    ctx->sp_clean_floats = ctx->sp_ent_words = ctx->sp_cnt_words = 0;
    hipError_t e;
    if ((e = hipMalloc((void**)&ctx->sp_clean, clean_floats * 4)) != hipSuccess ||
        (e = hipMalloc((void**)&ctx->sp_ent, ent_words * 4)) != hipSuccess ||
        (e = hipMalloc((void**)&ctx->sp_cnt, cnt_words * 4)) != hipSuccess) {
      (void)hipGetLastError();
      if (ctx->sp_clean) (void)hipFree(ctx->sp_clean);
      if (ctx->sp_ent) (void)hipFree(ctx->sp_ent);
      ctx->sp_clean = nullptr;
      ctx->sp_ent = ctx->sp_cnt = nullptr;
      return fail(ctx, DM_ENOMEM, "buffers of the sparse-correction option (%zu bytes) could not be allocated: %s",
                  clean_floats * 4 + ent_words * 4 + cnt_words * 4, hipGetErrorString(e));
    }
    ctx->sp_clean_floats = clean_floats;
    ctx->sp_ent_words = ent_words;
    ctx->sp_cnt_words = cnt_words;
  }
  // one undropped row per position: the same step with K = 1 and p = 0, every logit written (scale 1)
  dm_params cp = *prm;
  cp.K = 1;
  cp.p = 0.0f;
  cp.flags = 0;
  dm::RowGeom gc;
  if (dm_status st = make_geom(ctx, &cp, true, &gc)) return st;
  if (dm_status st = run_contraction(ctx, &cp, gc, true, h, W, ctx->sp_clean, 0, prm->V, s)) return st;
  hipError_t e = dm::launch_drop_lists(h, ctx->sp_ent, ctx->sp_cnt, ctx->keys, prm->seeds, g, s);
  if (e != hipSuccess) return fail_hip(ctx, "drop_lists launch", e);
  e = dm::launch_sparse_correct(W, ctx->sp_clean, ctx->sp_ent, ctx->sp_cnt, ctx->keys, (int)P, prm->K, prm->d, prm->V, s);
  if (e != hipSuccess) return fail_hip(ctx, "sparse_correct launch", e);
  return DM_OK;
}

// The verification step; draft_probs != nullptr selects the distribution-level rules.
dm_status verify_impl(dm_ctx* ctx, const dm_params* prm, const void* h, const void* W, const int32_t* draft_ids,
                      const float* draft_probs, int32_t* accept_len, int32_t* best_node, uint8_t* accept_mask,
                      uint8_t* hit, int32_t* path_ids, int32_t* vote_ids, int32_t* vote_cnt, float* js_draft,
                      float* js_heads, void* stream) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  if (!prm) return fail(ctx, DM_EINVAL, "params is NULL");
  if (!h || !W || !draft_ids || !accept_len) return fail(ctx, DM_EINVAL, "h, W, draft_ids and accept_len are required");
  if (((uintptr_t)h | (uintptr_t)W) & 15) return fail(ctx, DM_EINVAL, "h and W must be 16-byte aligned");
  const bool mfma = use_mfma(prm);
  dm::RowGeom g;
  if (dm_status st = make_geom(ctx, prm, mfma, &g)) return st;
  const bool js = draft_probs != nullptr;
  dm::JsGeom jg{};
  dm::LogitStore store{nullptr, 0, 0, 0, 0};
  if (js) {
    jg.P = prm->B * prm->T;
    jg.K = prm->K;
    jg.K4 = (int)round_up(prm->K, 4);
    jg.KU = g.clean_last ? prm->K - 1 : prm->K;
    jg.V = prm->V;
    jg.NC = (prm->V + dm::kJsChunk - 1) / dm::kJsChunk;
    jg.KS = jg.K4 + 4;
    if ((int64_t)prm->B * prm->T > 0x7FFFFFFF) return fail(ctx, DM_EINVAL, "B*T too large");
    // the contraction kernels address the logit store of one 256-row tile with 32-bit byte offsets
    if ((int64_t)(256 / prm->K + 2) * prm->V * jg.K4 * 4 >= ((int64_t)1 << 32))
      return fail(ctx, DM_EUNSUPPORTED, "V = %d is too large for the distribution-level rules with K = %d", prm->V, prm->K);
    if (!ctx->lt) return fail(ctx, DM_EINVAL, "call dm_reserve_js before dropmatch_verify_js");
    if ((size_t)jg.P * (size_t)jg.V * (size_t)jg.K4 > ctx->lt_floats ||
        (size_t)jg.P * (size_t)jg.NC * (size_t)jg.KS > ctx->part_floats)
      return fail(ctx, DM_EINVAL, "B*T = %d positions with K = %d exceed what dm_reserve_js reserved", jg.P, jg.K);
    store = dm::LogitStore{ctx->lt, jg.K, jg.K4, jg.V, g.clean_last};
  }
  const bool nucleus = !js && (prm->flags & DM_FLAG_SAMPLE_PATHS) && prm->top_p > 0.0f && prm->top_p < 1.0f;
  dm::NucGeom ng{};
  if (nucleus) {
    ng.P = prm->B * prm->T;
    ng.K = prm->K;
    ng.K4 = (int)round_up(prm->K, 4);
    ng.KP = 4;
    while (ng.KP < ng.K4) ng.KP *= 2;
    ng.KU = g.clean_last ? prm->K - 1 : prm->K;
    ng.V = prm->V;
    ng.cap = (int)ctx->nuc_cap;
    ng.fine = dm::nucleus_fine_bins(ng.KP, prm->temperature) ? 1 : 0;
    if ((int64_t)prm->B * prm->T > 0x7FFFFFFF) return fail(ctx, DM_EINVAL, "B*T too large");
    if ((int64_t)(256 / prm->K + 2) * prm->V * ng.K4 * 4 >= ((int64_t)1 << 32))
      return fail(ctx, DM_EUNSUPPORTED, "V = %d is too large for nucleus sampling with K = %d", prm->V, prm->K);
    if (!ctx->lt || !ctx->nuc.hist)
      return fail(ctx, DM_EINVAL, "nucleus sampling (0 < top_p < 1) keeps the logits: call dm_reserve_js first");
    if ((size_t)ng.P * (size_t)ng.V * (size_t)ng.K4 > ctx->lt_floats || (size_t)ng.P * (size_t)ng.K > ctx->nuc_rows)
      return fail(ctx, DM_EINVAL, "B*T = %d positions with K = %d exceed what dm_reserve_js reserved", ng.P, ng.K);
    store = dm::LogitStore{ctx->lt, ng.K, ng.K4, ng.V, g.clean_last};
  }
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, DM_EHIP, "cannot select device %d", ctx->device);
  hipStream_t s = static_cast<hipStream_t>(stream);

  hipEvent_t* ev = nullptr;
  if (ctx->prof_enabled && ctx->ev && ctx->prof_calls < DM_PROFILE_MAX_CALLS && (ctx->prof_seen++ % ctx->prof_stride) == 0)
    ev = ctx->ev + kEv * ctx->prof_calls;
  const bool all_stages = ctx->prof_enabled == 1;
  const int Kv = g.clean_last ? prm->K - 1 : prm->K;
  dm::VoteOut out{accept_len, best_node, accept_mask, hit, path_ids, vote_ids, vote_cnt, js_draft, js_heads};
  // token-level rules on the W-streaming kernel: the acceptance step runs as the tail of that launch
  dm::VoteFuse fuse{ctx->done, draft_ids, prm->parent, prm->B, prm->T, prm->K, Kv, prm->rule, out};
  const bool want_fuse = !js && !(prm->flags & DM_FLAG_SEPARATE_VOTE);
  bool fused = false;
  if (prm->flags & DM_FLAG_SPARSE_CORRECTION) {
    if (js || (prm->flags & (DM_FLAG_SAMPLE_PATHS | DM_FLAG_FORCE_GENERIC)) || !mfma || prm->K > dm::kSparseMaxK || ctx->borrowed)
      return fail(ctx, DM_EUNSUPPORTED, "DM_FLAG_SPARSE_CORRECTION takes bf16 with d %% 64 == 0, K <= %d, a token-level rule, "
                  "arg-max path tokens, on a context", dm::kSparseMaxK);
    if (dm_status st = run_sparse_correction(ctx, prm, g, h, W, s)) return st;
    const hipError_t ev_ = dm::launch_vote_accept(ctx->keys, draft_ids, prm->parent, prm->B, prm->T, prm->K, Kv, prm->rule, out,
                                                  nullptr, nullptr, s);
    if (ev_ != hipSuccess) return fail_hip(ctx, "vote_accept launch", ev_);
    return DM_OK;
  }
  // sampled tokens on the 256 x 256 kernel: its copy wavefronts leave a tile of noise (256 KB) per workgroup,
  // at most one workgroup per compute unit; allocated by the first call that needs it
  if ((prm->flags & DM_FLAG_SAMPLE_PATHS) && !nucleus && mfma && g.M > 128 && ctx->noise == nullptr && !ctx->borrowed) {
    const hipError_t ea = hipMalloc((void**)&ctx->noise, (size_t)ctx->num_cu * 256 * 256 * 4);
    if (ea != hipSuccess) {
      (void)hipGetLastError();
      ctx->noise = nullptr;
      return fail(ctx, DM_ENOMEM, "noise scratch of %zu bytes for sampled path tokens could not be allocated: %s "
                  "(the first such call allocates; make it outside a stream capture)",
                  (size_t)ctx->num_cu * 256 * 256 * 4, hipGetErrorString(ea));
    }
  }
  if (dm_status st = run_contraction(ctx, prm, g, mfma, h, W, nullptr, 0, 0, s, ev, store, want_fuse ? &fuse : nullptr,
                                     &fused, nucleus ? (int64_t)ng.P * ng.K : 0))
    return st;
  hipError_t e;
  if (js) {
    const float scale = (float)(1.0 / (1.0 - (double)prm->p));
    e = dm::launch_js_stats(ctx->lt, ctx->keys, ctx->part_a, jg, scale, s);
    if (e != hipSuccess) return fail_hip(ctx, "js_stats launch", e);
    if (ev && all_stages) (void)hipEventRecord(ev[3], s);
    e = dm::launch_js_terms(ctx->lt, ctx->keys, ctx->part_a, draft_probs, draft_ids, ctx->part_b, jg, scale, s);
    if (e != hipSuccess) return fail_hip(ctx, "js_terms launch", e);
    if (ev && all_stages) (void)hipEventRecord(ev[4], s);
  } else if (nucleus) {
    const float scale = (float)(1.0 / (1.0 - (double)prm->p));
    const dm::SampleCfg samp{ctx->seeds_dev, 0.f, prm->T, prm->K, prm->step, g.clean_last, nullptr, prm->step_dev};
    e = dm::launch_nucleus(ctx->lt, ctx->keys, ctx->nuc, ng, samp, scale, (float)(1.0 / (double)prm->temperature),
                           (double)prm->top_p, s);
    if (e != hipSuccess) return fail_hip(ctx, "nucleus launch", e);
    if (ev && all_stages) {  // reported in the two slots of the distribution-level passes
      (void)hipEventRecord(ev[3], s);
      (void)hipEventRecord(ev[4], s);
    }
  } else if (ev && all_stages) {
    (void)hipEventRecord(ev[3], s);
    (void)hipEventRecord(ev[4], s);
  }
  if (!fused) {
    e = dm::launch_vote_accept(nucleus ? ctx->nuc.keys_s : ctx->keys, draft_ids, prm->parent, prm->B, prm->T, prm->K, Kv, prm->rule, out,
                               js ? ctx->part_b : nullptr, js ? &jg : nullptr, s);
    if (e != hipSuccess) return fail_hip(ctx, "vote_accept launch", e);
  }
  if (ev) {
    if (all_stages) (void)hipEventRecord(ev[5], s);
    ctx->prof_kind[ctx->prof_calls] = (uint8_t)(((js || nucleus) ? 1 : 0) | (fused ? 0 : 2) | (js ? 4 : 0));
    ++ctx->prof_calls;
  }
  return DM_OK;
}

}  // namespace

extern "C" {

dm_status dm_validate(const dm_params* prm, char* msg, int32_t msg_len) {
  char scratch[128];
  const char* why = check_params(prm, scratch, sizeof scratch);
  if (msg && msg_len > 0) snprintf(msg, (size_t)msg_len, "%s", why ? why : "");
  return why ? DM_EINVAL : DM_OK;
}

int32_t dm_kernel_choice(const dm_params* prm) {
  char scratch[128];
  if (check_params(prm, scratch, sizeof scratch)) return DM_EINVAL;
  return use_mfma(prm) ? 1 : 0;
}

const char* dm_last_error(const dm_ctx* ctx) { return ctx ? ctx->err : g_err; }

dm_status dm_create(dm_ctx** out, int device, int64_t max_rows, int32_t max_d, int32_t max_V) {
  if (!out) return fail(nullptr, DM_EINVAL, "out is NULL");
  *out = nullptr;
  if (max_rows < 1 || max_d < 1 || max_V < 1) return fail(nullptr, DM_EINVAL, "max_rows, max_d, max_V must be >= 1");
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess) return fail_hip(nullptr, "hipGetDeviceCount", e);
  if (device < 0 || device >= ndev) return fail(nullptr, DM_EINVAL, "device %d not in 0..%d", device, ndev - 1);
  DeviceGuard guard(device);
  if (!guard.ok) return fail(nullptr, DM_EHIP, "cannot select device %d", device);

  hipDeviceProp_t prop;
  if ((e = hipGetDeviceProperties(&prop, device)) != hipSuccess) return fail_hip(nullptr, "hipGetDeviceProperties", e);
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return fail(nullptr, DM_EUNSUPPORTED, "device %d is %s; this library is built for gfx950 only", device, prop.gcnArchName);

  dm_ctx* ctx = new (std::nothrow) dm_ctx();
  if (!ctx) return fail(nullptr, DM_ENOMEM, "host allocation failed");
  ctx->device = device;
  ctx->num_cu = prop.multiProcessorCount;
  ctx->max_rows = max_rows;
  ctx->max_d = max_d;
  ctx->max_V = max_V;
  ctx->rows_pad = round_up(max_rows, 256);
  ctx->d_pad = (int32_t)round_up(max_d, 64);
  const size_t a_bytes = (size_t)ctx->rows_pad * (size_t)ctx->d_pad * 4;
  if ((e = hipMalloc(&ctx->a_ws, a_bytes)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->keys, (size_t)ctx->rows_pad * 8)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->done, 256)) != hipSuccess || (e = hipMemset(ctx->done, 0, 256)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->seeds_dev, (size_t)ctx->rows_pad * 8)) != hipSuccess) {
    (void)hipGetLastError();
    if (ctx->a_ws) (void)hipFree(ctx->a_ws);
    if (ctx->keys) (void)hipFree(ctx->keys);
    if (ctx->done) (void)hipFree(ctx->done);
    if (ctx->seeds_dev) (void)hipFree(ctx->seeds_dev);
    if (ctx->noise) (void)hipFree(ctx->noise);
    delete ctx;
    return fail(nullptr, DM_ENOMEM, "workspace allocation of %zu bytes failed: %s", a_bytes, hipGetErrorString(e));
  }
  if ((e = dm::prepare_lmhead_mfma()) != hipSuccess || (e = dm::prepare_lmhead_mfma_big()) != hipSuccess ||
      (e = dm::prepare_vote_accept()) != hipSuccess || (e = dm::prepare_nucleus()) != hipSuccess) {
    (void)hipFree(ctx->a_ws);
    (void)hipFree(ctx->keys);
    (void)hipFree(ctx->done);
    (void)hipFree(ctx->seeds_dev);
    if (ctx->noise) (void)hipFree(ctx->noise);
    delete ctx;
    return fail_hip(nullptr, "raising the dynamic LDS limit", e);
  }
  *out = ctx;
  return DM_OK;
}

dm_status dropmatch_verify_static(int device, const dm_params* prm, const void* h, const void* W,
                                  const int32_t* draft_ids, int32_t* accept_len, int32_t* best_node,
                                  uint8_t* accept_mask, uint8_t* hit, int32_t* path_ids, int32_t* vote_ids,
                                  int32_t* vote_cnt, void* stream) {
  dm_ctx* ctx = nullptr;
  if (dm_status st = static_context(device, &ctx)) return st;
  // limits of the fixed workspace, checked before anything is enqueued
  char scratch[128];
  if (const char* why = check_params(prm, scratch, sizeof scratch)) return fail(nullptr, DM_EINVAL, "%s", why);
  if (prm->rule >= DM_RULE_JS)
    return fail(nullptr, DM_EUNSUPPORTED, "dropmatch_verify_static takes the token-level rules only (the others keep every logit)");
  const int64_t M = (int64_t)prm->B * prm->T * prm->K;
  if (M > DM_STATIC_MAX_ROWS || prm->B > DM_STATIC_MAX_ROWS)
    return fail(nullptr, DM_EINVAL, "B*T*K = %lld exceeds DM_STATIC_MAX_ROWS = %d", (long long)M, DM_STATIC_MAX_ROWS);
  const bool mfma = use_mfma(prm);
  const int64_t M_pad = mfma ? (M <= 128 ? round_up(M, 32) : round_up(M, 256)) : round_up(M, 128);
  const int64_t ws = M_pad * round_up(prm->d, 64) * (prm->dtype == DM_BF16 ? 2 : 4);
  if (ws > (int64_t)DM_STATIC_MAX_WS_BYTES)
    return fail(nullptr, DM_EINVAL, "the masked rows of this call take %lld bytes, more than DM_STATIC_MAX_WS_BYTES = %d",
                (long long)ws, DM_STATIC_MAX_WS_BYTES);
  if ((prm->flags & DM_FLAG_SAMPLE_PATHS) && prm->top_p > 0.0f && prm->top_p < 1.0f)
    return fail(nullptr, DM_EUNSUPPORTED, "dropmatch_verify_static does not sample from a nucleus (that keeps every logit)");
  // (sampled path tokens on more than 128 rows draw their noise in the epilogue here: the noise buffer
  // of the faster variant is not part of the fixed workspace)
  const dm_status st = verify_impl(ctx, prm, h, W, draft_ids, nullptr, accept_len, best_node, accept_mask, hit, path_ids,
                                   vote_ids, vote_cnt, nullptr, nullptr, stream);
  if (st != DM_OK) snprintf(g_err, sizeof g_err, "%s", ctx->err);
  return st;
}

dm_status dm_destroy(dm_ctx* ctx) {
  if (!ctx) return DM_OK;
  DeviceGuard guard(ctx->device);
  dm_status st = DM_OK;
  if (!guard.ok || hipDeviceSynchronize() != hipSuccess) st = fail(nullptr, DM_EHIP, "device synchronisation failed in dm_destroy");
  drop_events(ctx);
  if (ctx->a_ws) (void)hipFree(ctx->a_ws);
  if (ctx->keys) (void)hipFree(ctx->keys);
  if (ctx->done) (void)hipFree(ctx->done);
  if (ctx->seeds_dev) (void)hipFree(ctx->seeds_dev);
  if (ctx->noise) (void)hipFree(ctx->noise);
  if (ctx->sp_clean) (void)hipFree(ctx->sp_clean);
  if (ctx->sp_ent) (void)hipFree(ctx->sp_ent);
  if (ctx->sp_cnt) (void)hipFree(ctx->sp_cnt);
  if (ctx->lt) (void)hipFree(ctx->lt);
  if (ctx->part_a) (void)hipFree(ctx->part_a);
  if (ctx->part_b) (void)hipFree(ctx->part_b);
  free_nucleus(ctx);
  delete ctx;
  return st;
}

dm_status dropmatch_verify(dm_ctx* ctx, const dm_params* prm, const void* h, const void* W,
                           const int32_t* draft_ids, int32_t* accept_len, int32_t* best_node,
                           uint8_t* accept_mask, uint8_t* hit, int32_t* path_ids, int32_t* vote_ids,
                           int32_t* vote_cnt, void* stream) {
  if (ctx && prm && prm->rule >= DM_RULE_JS)
    return fail(ctx, DM_EINVAL, "rules DM_RULE_JS and DM_RULE_JS_OR_MAJORITY need the draft distribution: call dropmatch_verify_js");
  return verify_impl(ctx, prm, h, W, draft_ids, nullptr, accept_len, best_node, accept_mask, hit, path_ids, vote_ids,
                     vote_cnt, nullptr, nullptr, stream);
}

dm_status dropmatch_verify_js(dm_ctx* ctx, const dm_params* prm, const void* h, const void* W,
                              const int32_t* draft_ids, const float* draft_probs, int32_t* accept_len,
                              int32_t* best_node, uint8_t* accept_mask, uint8_t* hit, int32_t* path_ids,
                              int32_t* vote_ids, int32_t* vote_cnt, float* js_draft, float* js_heads,
                              void* stream) {
  if (ctx && prm && prm->rule < DM_RULE_JS)
    return fail(ctx, DM_EINVAL, "dropmatch_verify_js takes DM_RULE_JS or DM_RULE_JS_OR_MAJORITY");
  if (ctx && !draft_probs) return fail(ctx, DM_EINVAL, "draft_probs is required");
  return verify_impl(ctx, prm, h, W, draft_ids, draft_probs, accept_len, best_node, accept_mask, hit, path_ids,
                     vote_ids, vote_cnt, js_draft, js_heads, stream);
}

dm_status dm_reserve_js(dm_ctx* ctx, int64_t max_positions, int32_t max_K) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  if (max_positions < 1 || max_K < 1 || max_K > DM_MAX_K_JS)
    return fail(ctx, DM_EINVAL, "need max_positions >= 1 and 1 <= max_K <= %d", DM_MAX_K_JS);
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, DM_EHIP, "cannot select device %d", ctx->device);
  if (hipDeviceSynchronize() != hipSuccess) return fail(ctx, DM_EHIP, "device synchronisation failed in dm_reserve_js");
  if (ctx->lt) (void)hipFree(ctx->lt);
  if (ctx->part_a) (void)hipFree(ctx->part_a);
  if (ctx->part_b) (void)hipFree(ctx->part_b);
  ctx->lt = ctx->part_a = ctx->part_b = nullptr;
  ctx->lt_floats = ctx->part_floats = 0;
  free_nucleus(ctx);
  const size_t K4 = (size_t)round_up(max_K, 4);
  const size_t lt_floats = (size_t)max_positions * (size_t)ctx->max_V * K4;
  const size_t nc = (size_t)((ctx->max_V + dm::kJsChunk - 1) / dm::kJsChunk);
  const size_t part_floats = (size_t)max_positions * nc * (K4 + 4);
  hipError_t e;
  if ((e = hipMalloc((void**)&ctx->lt, lt_floats * 4)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->part_a, part_floats * 4)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->part_b, part_floats * 4)) != hipSuccess) {
    (void)hipGetLastError();
    if (ctx->lt) (void)hipFree(ctx->lt);
    if (ctx->part_a) (void)hipFree(ctx->part_a);
    ctx->lt = ctx->part_a = ctx->part_b = nullptr;
    return fail(ctx, DM_ENOMEM, "logit store of %zu bytes could not be allocated: %s", lt_floats * 4, hipGetErrorString(e));
  }
  ctx->lt_floats = lt_floats;
  ctx->part_floats = part_floats;
  // nucleus sampling: 512 digit bins (coarse, fine) of 8 bytes per row, kept zero between calls
  const size_t rows = (size_t)max_positions * (size_t)max_K;
  const int64_t cap = dm::nucleus_list_capacity(ctx->max_V);
  if ((e = hipMalloc((void**)&ctx->nuc.hist, rows * 512 * 8)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->nuc.digit0, rows * 4)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->nuc.cand_n, rows * 4)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->nuc.cand, rows * (size_t)cap * 8)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->nuc.below, rows * 8)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->nuc.target, rows * 8)) != hipSuccess ||
      (e = hipMalloc((void**)&ctx->nuc.keys_s, rows * 8)) != hipSuccess ||
      (e = hipMemset(ctx->nuc.hist, 0, rows * 512 * 8)) != hipSuccess) {
    (void)hipGetLastError();
    free_nucleus(ctx);
    return fail(ctx, DM_ENOMEM, "nucleus buffers for %zu rows could not be allocated: %s", rows, hipGetErrorString(e));
  }
  ctx->nuc_rows = rows;
  ctx->nuc_cap = cap;
  return DM_OK;
}

dm_status dm_set_profiling(dm_ctx* ctx, int32_t enabled) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, DM_EHIP, "cannot select device %d", ctx->device);
  ctx->prof_calls = 0;
  ctx->prof_seen = 0;
  ctx->prof_enabled = 0;
  if (!enabled) return DM_OK;
  if (!ctx->ev) {
    ctx->ev = new (std::nothrow) hipEvent_t[kEv * DM_PROFILE_MAX_CALLS]();
    if (!ctx->ev) return fail(ctx, DM_ENOMEM, "host allocation failed");
    for (int i = 0; i < kEv * DM_PROFILE_MAX_CALLS; ++i) {
      const hipError_t e = hipEventCreate(&ctx->ev[i]);
      if (e != hipSuccess) {
        drop_events(ctx);
        return fail_hip(ctx, "hipEventCreate", e);
      }
    }
  }
  ctx->prof_enabled = enabled == 2 ? 2 : 1;
  return DM_OK;
}

dm_status dm_set_profiling_stride(dm_ctx* ctx, int32_t stride) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  if (stride < 1) return fail(ctx, DM_EINVAL, "stride must be at least 1, got %d", stride);
  ctx->prof_stride = stride;
  return DM_OK;
}

dm_status dm_get_profile_stages(dm_ctx* ctx, int32_t* n_calls, float* ms /* [5] */) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, DM_EHIP, "cannot select device %d", ctx->device);
  const int n = ctx->prof_calls;
  double sum[kEv - 1] = {0, 0, 0, 0, 0};
  if (n > 0) {
    const bool light = ctx->prof_enabled == 2;  // only events 1 and 2 of every call exist
    hipError_t e = hipEventSynchronize(ctx->ev[kEv * (n - 1) + (light ? 2 : kEv - 1)]);
    if (e != hipSuccess) return fail_hip(ctx, "hipEventSynchronize", e);
    for (int c = 0; c < n; ++c)
      for (int k = light ? 1 : 0; k < (light ? 2 : kEv - 1); ++k) {
        // a bracket with no kernel inside would read the cost of an event pair (a few microseconds)
        if (k == 2 && !(ctx->prof_kind[c] & 1)) continue;
        if (k == 3 && !(ctx->prof_kind[c] & 4)) continue;
        if (k == 4 && !(ctx->prof_kind[c] & 2)) continue;
        float t = 0.f;
        e = hipEventElapsedTime(&t, ctx->ev[kEv * c + k], ctx->ev[kEv * c + k + 1]);
        if (e != hipSuccess) return fail_hip(ctx, "hipEventElapsedTime", e);
        sum[k] += t;
      }
  }
  if (n_calls) *n_calls = n;
  if (ms)
    for (int k = 0; k < kEv - 1; ++k) ms[k] = n ? (float)(sum[k] / n) : 0.f;
  return DM_OK;
}

dm_status dm_get_profile_samples(dm_ctx* ctx, int32_t stage, float* ms, int32_t n_max, int32_t* n_out) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  if (stage < 0 || stage >= kEv - 1 || !ms || n_max < 0 || !n_out) return fail(ctx, DM_EINVAL, "need 0 <= stage < 5, ms, n_max >= 0, n_out");
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, DM_EHIP, "cannot select device %d", ctx->device);
  const bool light = ctx->prof_enabled == 2;  // only events 1 and 2 of every call exist
  *n_out = 0;
  if (light && stage != 1) return DM_OK;
  const int n = ctx->prof_calls;
  if (n > 0) {
    const hipError_t e = hipEventSynchronize(ctx->ev[kEv * (n - 1) + (light ? 2 : kEv - 1)]);
    if (e != hipSuccess) return fail_hip(ctx, "hipEventSynchronize", e);
  }
  for (int c = 0; c < n && *n_out < n_max; ++c) {
    if (stage == 2 && !(ctx->prof_kind[c] & 1)) continue;
    if (stage == 3 && !(ctx->prof_kind[c] & 4)) continue;
    if (stage == 4 && !(ctx->prof_kind[c] & 2)) continue;
    float t = 0.f;
    const hipError_t e = hipEventElapsedTime(&t, ctx->ev[kEv * c + stage], ctx->ev[kEv * c + stage + 1]);
    if (e != hipSuccess) return fail_hip(ctx, "hipEventElapsedTime", e);
    ms[(*n_out)++] = t;
  }
  return DM_OK;
}

dm_status dm_get_profile(dm_ctx* ctx, int32_t* n_calls, float* ms_mask, float* ms_lmhead, float* ms_vote) {
  float ms[kEv - 1];
  if (dm_status st = dm_get_profile_stages(ctx, n_calls, ms)) return st;
  if (ms_mask) *ms_mask = ms[0];
  if (ms_lmhead) *ms_lmhead = ms[1];
  if (ms_vote) *ms_vote = ms[4];
  return DM_OK;
}

dm_status dm_debug_masks(dm_ctx* ctx, const dm_params* prm, uint32_t* bits, void* stream) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  if (!prm || !bits) return fail(ctx, DM_EINVAL, "params and bits are required");
  dm::RowGeom g;
  if (dm_status st = make_geom(ctx, prm, false, &g)) return st;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, DM_EHIP, "cannot select device %d", ctx->device);
  hipError_t e = dm::launch_mask_bits(bits, prm->seeds, g, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(ctx, "mask_bits launch", e);
  return DM_OK;
}

dm_status dm_debug_stream_read(dm_ctx* ctx, const void* src, int64_t bytes, void* stream) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  if (!src || bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15))
    return fail(ctx, DM_EINVAL, "need a 16-byte aligned buffer of a positive multiple of 16 bytes");
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, DM_EHIP, "cannot select device %d", ctx->device);
  const hipError_t e = dm::launch_stream_read(src, (size_t)bytes, ctx->num_cu, ctx->done + 32, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(ctx, "stream_read launch", e);
  return DM_OK;
}

dm_status dm_debug_logits(dm_ctx* ctx, const dm_params* prm, const void* h, const void* W, int32_t v0,
                          int32_t v1, float* logits, void* stream) {
  if (!ctx) return fail(nullptr, DM_EINVAL, "ctx is NULL");
  if (!prm || !h || !W || !logits) return fail(ctx, DM_EINVAL, "params, h, W and logits are required");
  if (((uintptr_t)h | (uintptr_t)W) & 15) return fail(ctx, DM_EINVAL, "h and W must be 16-byte aligned");
  const bool mfma = use_mfma(prm);
  dm::RowGeom g;
  if (dm_status st = make_geom(ctx, prm, mfma, &g)) return st;
  if (v0 < 0 || v1 <= v0 || v1 > prm->V) return fail(ctx, DM_EINVAL, "need 0 <= v0 < v1 <= V");
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, DM_EHIP, "cannot select device %d", ctx->device);
  return run_contraction(ctx, prm, g, mfma, h, W, logits, v0, v1, static_cast<hipStream_t>(stream));
}

}  // extern "C"
