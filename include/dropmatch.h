/*
 * dropmatch.h - C ABI of the DropMatch Monte-Carlo-dropout LM-head verification step
 * for AMD Instinct MI355X (gfx950).
 *
 * The step (paper: Methodology, "Multi-Sample LM Head via MC Dropout" and "Acceptance
 * Criteria"): for every row t of the final hidden states h, draw K keep-masks
 * m^(i) ~ Bernoulli(1 - p_drop)^d (Eq. 1), form h_t^(i) = h_t * m^(i) / (1 - p_drop)
 * (Eq. 2), project through the shared LM head, l_t^(i) = W h_t^(i) (Eq. 3), reduce each
 * path to its token y_t^(i) = argmax_v l_t^(i)[v], and accept the draft token of the row
 * if it is one of the K path tokens (Eq. 4, naive token matching) or if it is their
 * most frequent token (Eq. 7, majority).  The first rejected row rejects all later ones;
 * the number of accepted draft tokens is the accepted length.  With draft trees (the
 * EAGLE-3 experiments use tree decoding with naive matching) the rule is applied along
 * parent links and the result is the depth of the deepest accepted node.
 *
 * Everything here is plain C: opaque context, plain pointers, sizes.  Pointers are
 * marked HOST or DEVICE.  The caller owns every buffer it passes; the library owns only
 * the workspace inside the context, allocates nothing per call, never synchronises the
 * stream and never frees caller memory.  All device work is enqueued on the stream the
 * caller passes (a hipStream_t cast to void*; NULL is the default stream).
 *
 * Errors: every function returns a dm_status; DM_OK is 0, errors are negative.  A
 * failed call enqueues nothing.  dm_last_error() returns a human-readable message for
 * the last failure on that context (or, with NULL, of the last failed call that had no
 * context).  Faults inside kernels (e.g. a wrong DEVICE pointer) surface at the caller's
 * next synchronisation, as with any HIP launch.
 *
 * Random source (the paper only says "i.i.d. Bernoulli"): Philox4x32-10, counter
 * (j >> 2, row t, path i, step), key (low, high word of the sequence's 64-bit seed);
 * dimension j uses output word j & 3 and is kept iff word >= floor(p * 2^32).  Masks are
 * therefore a pure function of (seed, step, i, t, j): reproducible on any machine.
 */
#ifndef DROPMATCH_H
#define DROPMATCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dm_ctx dm_ctx; /* opaque; owns only its workspace */

typedef enum {
  DM_OK = 0,
  DM_EINVAL = -1,       /* bad argument (null pointer, size, p, enum, limit of the context) */
  DM_ENOMEM = -2,       /* workspace allocation failed in dm_create */
  DM_EHIP = -3,         /* a HIP runtime call failed; message holds hipGetErrorString */
  DM_EUNSUPPORTED = -4  /* valid request outside what this build implements */
} dm_status;

typedef enum { DM_F32 = 0, DM_BF16 = 1 } dm_dtype; /* storage type of BOTH h and W */

typedef enum {
  DM_RULE_ANY = 0,            /* Eq. 4: draft token is among the K path tokens */
  DM_RULE_MAJORITY = 1,       /* Eq. 7: draft token equals the mode of the K path tokens */
  DM_RULE_JS = 2,             /* Eq. 6 alone: JS(draft dist. || centroid) <= max_i JS(head i || centroid) */
  DM_RULE_JS_OR_MAJORITY = 3  /* Algorithm 1: Eq. 6, else Eq. 7 */
} dm_rule;                    /* rules 2 and 3 go through dropmatch_verify_js */

/* One mask per path shared by all rows of a sequence ("K persistent heads"): the row word
 * of the Philox counter is forced to 0.  Default (flag clear): a fresh mask per (path, row). */
#define DM_FLAG_SHARE_MASK_ACROSS_POS 1u
/* Testing aid: run the contraction on the generic fp32-FMA kernel even where the MFMA
 * kernel applies (lets the two kernels be compared on the same inputs). */
#define DM_FLAG_FORCE_GENERIC 2u

/* Path K-1 of every row is computed without dropout (all dimensions kept, no 1/(1-p)): the plain
 * LM head.  Its token, the greedy target token of the row, is returned in path_ids[b,t,K-1] (the
 * token to emit after a rejection or as the bonus token; the paper leaves that choice open), and
 * the rules (Eq. 4, 6, 7, Algorithm 1), vote_ids/vote_cnt and js_heads use paths 0..K-2 only
 * (js_heads[b,t,K-1] = 0).  The masks of the other paths are those of a call without the flag.
 * Needs K >= 2. */
#define DM_FLAG_CLEAN_LAST_PATH 4u

/* Sampled path tokens.  The paper remarks that the token of a path may be "selected by nucleus
 * sampling" instead of being the arg max, without giving parameters.  With this flag the token of path
 * i at row t is a draw from Softmax(l_t^(i) / temperature), made by the Gumbel-max construction so that
 * it is a pure function of (seed, step, i, t): y = argmax_v (l[v] / temperature + g[v]),
 * g[v] = -ln(-ln u[v]), u[v] = ((w >> 9) + 1/2) 2^-23, w = word (v & 3) of Philox4x32-10 with counter
 * (v >> 2, t, i, step) and key = seed + 0x9E3779B97F4A7C15 (mod 2^64; a stream apart from the masks').
 * Ties -> smallest v.  Needs prm->temperature > 0; token-level rules only (dropmatch_verify); a
 * clean last path stays arg max.
 * With 0 < prm->top_p < 1 the arg max runs over the nucleus of that distribution only (Holtzman et
 * al.'s top-p set): most probable tokens first until their probabilities add up to top_p, tokens
 * as probable as the last one included; same noise, so the draw follows the distribution
 * renormalised on the set and top_p -> 1 gives the unrestricted draw.  This variant keeps the
 * logits of the call (dm_reserve_js must have been called for B*T positions and K paths;
 * K <= DM_MAX_K_JS, T*K <= DM_MAX_TK_JS), finds each row's threshold (with t the distance from the
 * row's maximum over the temperature: probability mass in 64-bit integers, floor(e^-t 2^44), so
 * reproducible run to run; tokens whose t agree to 2^-19 count as equally probable) and then draws
 * from the stored logits.  Rows whose distribution is so flat that more than an eighth of the
 * vocabulary lies within 0.125 of the threshold in t (1/128 from temperature 2 on, up to 32 paths)
 * take a slower path through the logit store: same result, several times the time. */
#define DM_FLAG_SAMPLE_PATHS 16u

/* The same path logits by linearity of Eq. 3, W (h * m) = W h - W (h * (1 - m)): one undropped row per
 * position on the matrix cores plus, per path, a correction over the dimensions that path dropped, on the
 * vector ALU.  Same tokens as the default path up to the order of the float32 sums.  Measured slower than
 * the dense contraction on this chip at the paper's dropout rates; kept as an option.  bf16 with d % 64 == 0,
 * K <= 32, token-level rules, arg-max path tokens.  The first call with this flag allocates its buffers
 * (B*T*V*4 + B*T*K*d*4.07 bytes; later calls with larger shapes reallocate): make it outside a stream
 * capture.  DM_EUNSUPPORTED otherwise. */
#define DM_FLAG_SPARSE_CORRECTION 32u

/* Testing aid: always run the acceptance step as its own kernel.  (Without it, calls that go to the
 * W-streaming kernel - bf16, at most 128 masked rows, token-level rule - run that step inside the
 * contraction launch, in the workgroup that finishes last.) */
#define DM_FLAG_SEPARATE_VOTE 8u

/* Limits of this build. */
#define DM_MAX_K 1024            /* paths per row */
#define DM_MAX_ROWS_PER_SEQ 4096 /* T */
#define DM_MAX_TK 16384          /* T*K per sequence (path tokens of a sequence live in LDS) */
#define DM_MAX_K_JS 64           /* paths per row with the distribution-level rules */
#define DM_MAX_TK_JS 8192        /* T*K per sequence with the distribution-level rules */

typedef struct {
  int32_t B;       /* sequences, >= 1 */
  int32_t T;       /* rows of h per sequence: chain positions (incl. a bonus row) or tree nodes */
  int32_t K;       /* dropout paths per row, 1..DM_MAX_K */
  int32_t d;       /* hidden size */
  int32_t V;       /* vocabulary size */
  int32_t dtype;   /* dm_dtype */
  float p;         /* p_drop, 0 <= p < 1 (Eq. 1) */
  uint32_t step;   /* Philox counter word 3: vary per decode step to get fresh masks from fixed seeds.
                      seeds and step are read on the host and travel as kernel arguments: a call
                      captured into a HIP graph replays the masks (and sampling noise) it was
                      captured with; see step_dev for replays with fresh masks */
  int32_t rule;    /* dm_rule */
  uint32_t flags;  /* DM_FLAG_* */
  const uint64_t* seeds; /* HOST [B]: mask seed per sequence; read before the call returns */
  const int32_t* parent; /* DEVICE [B,T] or NULL.  NULL: chain.  Else tree: parent[b,0] = -1,
                            0 <= parent[b,n] < n.  A node whose parent index breaks this is
                            treated as rejected (never read out of bounds). */
  float temperature;     /* DM_FLAG_SAMPLE_PATHS only: > 0, finite.  Ignored otherwise. */
  float top_p;           /* DM_FLAG_SAMPLE_PATHS only: 0 or 1 = draw from the whole distribution;
                            0 < top_p < 1 = from its nucleus (see the flag).  Ignored otherwise. */
  const uint32_t* step_dev; /* DEVICE or NULL.  If given, the 32-bit word it points to is read by the kernels
                            when they RUN and added to `step` (mod 2^32): a call captured into a HIP graph
                            then draws fresh masks (and sampling noise) on every replay for which the
                            caller has changed that word, e.g. with a copy node or a one-thread kernel
                            ordered before the replay.  The word must stay valid and unchanged while the
                            call's kernels run. */
} dm_params;

/* Create a context on HIP device `device` able to serve calls with B*T*K <= max_rows,
 * d <= max_d, V <= max_V.  Allocates the workspace (masked rows: max_rows rounded up to
 * 256 times max_d rounded up to 64 elements of 4 bytes, plus 16 bytes per row).  One more buffer is
 * allocated later, by the first dropmatch_verify with DM_FLAG_SAMPLE_PATHS on more than 128 rows:
 * 256 KB per compute unit, 64 MB on an MI355X, for the noise of sampled path tokens (make that first
 * call outside a stream capture).  The context
 * may be used from one host thread at a time; calls on one context must be enqueued on
 * one stream (or be ordered by the caller), since they share the workspace. */
dm_status dm_create(dm_ctx** out, int device, int64_t max_rows, int32_t max_d, int32_t max_V);

/* Synchronises the device, frees the workspace and the context.  NULL is accepted. */
dm_status dm_destroy(dm_ctx* ctx);

/* Message of the last failure (string owned by the context / the library; never free it). */
const char* dm_last_error(const dm_ctx* ctx);

/* Pure host check of a parameter block (no device is touched; usable without a GPU):
 * sizes, p, enums, flags, limits, seeds != NULL.  `msg`/`msg_len` may be NULL/0; otherwise
 * receives a NUL-terminated reason on failure. */
dm_status dm_validate(const dm_params* prm, char* msg, int32_t msg_len);

/*
 * The verification step (Eq. 1-4 and 7, prefix / tree rule).  Rows are ordered (b, t, i):
 * row index = (b*T + t)*K + i.
 *
 * Chain mode (prm->parent == NULL): the K paths of row t test draft_ids[b,t].
 *   hit[b,t]        = rule(draft_ids[b,t], path_ids[b,t,:])
 *   accept_len[b]   = first t with hit == 0 (T if none)
 *   accept_mask[b,t]= 1 for t < accept_len[b], else 0
 *   best_node[b]    = accept_len[b] - 1
 *   A row with draft id < 0 (e.g. the bonus row after gamma draft tokens) never hits.
 * Tree mode: row n holds the hidden state of node n and predicts n's children.
 *   hit[b,0] = 1; hit[b,n] = rule(draft_ids[b,n], path_ids[b,parent[n],:]) for n > 0
 *   accept_mask[b,n] = hit[b,n] and accept_mask[b,parent[n]]
 *   accept_len[b]   = largest depth of an accepted node; best_node[b] = that node
 *                     (smallest index among equally deep ones)
 * In both modes vote_ids/vote_cnt give the mode of the K path tokens of every row and its
 * multiplicity (ties between modes: smallest token id); argmax ties: smallest vocabulary id.
 *
 * The LM-head product runs in the storage type with fp32 accumulation (bf16 x bf16 products
 * are exact in fp32); the K*T x V logits are never written to memory.  The factor
 * 1 / (1 - p) of Eq. 2 is positive and common to a row, so it cannot change an argmax and is
 * not applied on this path (dm_debug_logits applies it).
 *
 * h, W must be 16-byte aligned.  Inputs must be finite.
 */
dm_status dropmatch_verify(dm_ctx* ctx, const dm_params* prm,
                           const void* h,            /* DEVICE [B,T,d] contiguous */
                           const void* W,            /* DEVICE [V,d] row-major contiguous */
                           const int32_t* draft_ids, /* DEVICE [B,T] */
                           int32_t* accept_len,      /* DEVICE [B], required */
                           int32_t* best_node,       /* DEVICE [B] or NULL */
                           uint8_t* accept_mask,     /* DEVICE [B,T] or NULL */
                           uint8_t* hit,             /* DEVICE [B,T] or NULL */
                           int32_t* path_ids,        /* DEVICE [B,T,K] or NULL */
                           int32_t* vote_ids,        /* DEVICE [B,T] or NULL */
                           int32_t* vote_cnt,        /* DEVICE [B,T] or NULL */
                           void* stream);

/*
 * Distribution-level acceptance (paper: "JS-Divergence-Based Criterion", Eq. 5, Eq. 6, Algorithm 1).
 * With p_t^(i) = Softmax(l_t^(i)) (Eq. 3; here the factor 1/(1-p) of Eq. 2 IS applied, softmax is
 * not scale invariant), the centroid pbar_t = Softmax((1/K) sum_i l_t^(i)) (Eq. 5) and the draft
 * model's distribution phat_t, row t hits iff
 *     JS(phat_t || pbar_t) <= max_i JS(p_t^(i) || pbar_t)                        (Eq. 6, rule DM_RULE_JS)
 * or, under DM_RULE_JS_OR_MAJORITY (Algorithm 1), iff Eq. 6 holds or else Eq. 7 holds.
 * JS(P||Q) = KL(P||M)/2 + KL(Q||M)/2, M = (P+Q)/2, natural logarithm, 0 ln 0 = 0; both sides of
 * Eq. 6 are compared as float.  Chains only (prm->parent must be NULL; the paper pairs tree decoding
 * with naive matching only), K <= DM_MAX_K_JS, T*K <= DM_MAX_TK_JS.  A row with draft id < 0 never hits.
 *
 * dm_reserve_js allocates, once, what these rules need beyond dm_create: the logits of every path
 * (max_positions * max_V * roundup(max_K, 4) floats; unlike on the token-level path they are stored,
 * because Eq. 6 needs the normalisers before it can form its sums), two small arrays of partial
 * sums, and for nucleus sampling 2 KB of search state plus a candidate list of max(1024, max_V / 8)
 * (logit, token) pairs per masked row (max_positions * max_K rows; a quarter of the logit store at
 * K = 16).  It synchronises the device and may be called again to resize.  B*T <= max_positions and
 * K <= max_K must then hold for every dropmatch_verify_js on this context.
 *
 * dropmatch_verify_js: same contract and outputs as dropmatch_verify, plus
 *   draft_probs  DEVICE float [B,T,V]: phat of the token that row t verifies (probabilities, >= 0,
 *                summing to 1; exact zeros are allowed; ignored at rows with draft id < 0)
 *   js_draft     DEVICE float [B,T] or NULL: JS(phat_t || pbar_t); -1 at rows with draft id < 0
 *   js_heads     DEVICE float [B,T,K] or NULL: JS(p_t^(i) || pbar_t)
 * Arithmetic: logits from the same contraction kernels (storage type products, fp32 accumulation,
 * times (float)(1/(1-p))), exp/log and all sums in fp32 with partial sums added in a fixed order
 * (chunk totals in double), so results are reproducible run to run.
 */
dm_status dm_reserve_js(dm_ctx* ctx, int64_t max_positions, int32_t max_K);
dm_status dropmatch_verify_js(dm_ctx* ctx, const dm_params* prm,
                              const void* h,            /* DEVICE [B,T,d] contiguous */
                              const void* W,            /* DEVICE [V,d] row-major contiguous */
                              const int32_t* draft_ids, /* DEVICE [B,T] */
                              const float* draft_probs, /* DEVICE [B,T,V] */
                              int32_t* accept_len,      /* DEVICE [B], required */
                              int32_t* best_node,       /* DEVICE [B] or NULL */
                              uint8_t* accept_mask,     /* DEVICE [B,T] or NULL */
                              uint8_t* hit,             /* DEVICE [B,T] or NULL */
                              int32_t* path_ids,        /* DEVICE [B,T,K] or NULL */
                              int32_t* vote_ids,        /* DEVICE [B,T] or NULL */
                              int32_t* vote_cnt,        /* DEVICE [B,T] or NULL */
                              float* js_draft,          /* DEVICE [B,T] or NULL */
                              float* js_heads,          /* DEVICE [B,T,K] or NULL */
                              void* stream);

/*
 * dropmatch_verify without a context and without any allocation, for callers that cannot allocate
 * device memory: code that runs under a HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same step, same arguments and outputs as dropmatch_verify (token-level rules), with
 * the HIP device number in place of the context.  Its workspace (masked rows, argmax keys, seeds,
 * election counter) is a fixed array in device memory that is part of the library's code object:
 * DM_STATIC_MAX_WS_BYTES + 16 bytes per row of DM_STATIC_MAX_ROWS + 256 bytes, about 8 MB, held by
 * every GPU the library runs on until the process ends.  Nothing is allocated or freed, by this
 * function or by anything it calls; nothing is synchronised.
 * Limits (DM_EINVAL beyond them, nothing enqueued): B*T*K <= DM_STATIC_MAX_ROWS, and the masked rows
 * must fit: roundup(B*T*K, 32 if B*T*K <= 128 [bf16, d % 64 == 0] else 256 [same] else 128) *
 * roundup(d, 64) * (2 for bf16, 4 for f32) <= DM_STATIC_MAX_WS_BYTES (e.g. 1024 rows at d = 4096 in
 * bf16).  DM_EUNSUPPORTED for the distribution-level rules and nucleus sampling (those need buffers
 * that grow with the call; use a context).
 * The first call on a device looks up the array's address and the device's properties (no allocation
 * either, but make it outside a stream capture); later calls only enqueue kernels.
 * All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different streams
 * without ordering, several host threads) race and must be ordered by the caller.  What a call needs
 * to start from zero it clears itself, so an earlier call's contents never matter.
 * Messages of failures: dm_last_error(NULL), per host thread.
 */
#define DM_STATIC_MAX_ROWS 2048
#define DM_STATIC_MAX_WS_BYTES (8 * 1024 * 1024)
dm_status dropmatch_verify_static(int device, const dm_params* prm,
                                  const void* h,            /* DEVICE [B,T,d] contiguous */
                                  const void* W,            /* DEVICE [V,d] row-major contiguous */
                                  const int32_t* draft_ids, /* DEVICE [B,T] */
                                  int32_t* accept_len,      /* DEVICE [B], required */
                                  int32_t* best_node,       /* DEVICE [B] or NULL */
                                  uint8_t* accept_mask,     /* DEVICE [B,T] or NULL */
                                  uint8_t* hit,             /* DEVICE [B,T] or NULL */
                                  int32_t* path_ids,        /* DEVICE [B,T,K] or NULL */
                                  int32_t* vote_ids,        /* DEVICE [B,T] or NULL */
                                  int32_t* vote_cnt,        /* DEVICE [B,T] or NULL */
                                  void* stream);

/* Debug: the keep-masks of Eq. 1 exactly as dropmatch_verify draws them, bit-packed.
 * bits: DEVICE uint32 [B,T,K,ceil(d/32)]; word w of a row holds dimensions 32w..32w+31,
 * bit (j & 31) = keep(j); bits past d are 0. */
dm_status dm_debug_masks(dm_ctx* ctx, const dm_params* prm, uint32_t* bits, void* stream);

/* Debug: logits of Eq. 3 including the Eq. 2 scale, for vocabulary rows v0 <= v < v1, taken
 * from the accumulators of the same contraction kernel the verify path would use:
 * logits: DEVICE float [B*T*K, v1 - v0], value = (float)(1/(1-p)) * fp32 accumulator. */
dm_status dm_debug_logits(dm_ctx* ctx, const dm_params* prm, const void* h, const void* W,
                          int32_t v0, int32_t v1, float* logits, void* stream);

/* Measurement aid: enqueue a bare streaming read of `bytes` bytes (a positive multiple of 16, src 16-byte
 * aligned) of DEVICE memory, every byte once and nothing else.  Timed by the caller, it gives the read
 * bandwidth this machine delivers to a plain kernel: the achievable ceiling to quote beside the published HBM
 * peak for the kernels that are bound by streaming W (Eq. 3 at few masked rows). */
dm_status dm_debug_stream_read(dm_ctx* ctx, const void* src, int64_t bytes, void* stream);

/* Measurement aid.  dm_set_profiling(ctx, 1) makes every following dropmatch_verify /
 * dropmatch_verify_js record HIP events on its stream before and after each of its kernels
 * (mask rows, LM-head contraction + argmax, [JS pass 1, JS pass 2,] vote/accept); events are
 * created here, not in the verify calls.  At most DM_PROFILE_MAX_CALLS calls are kept (later
 * ones are not recorded).  dm_get_profile waits for the last recorded event and returns the
 * number of recorded calls and the mean duration of the three kernels of the token-level path
 * in milliseconds (any output pointer may be NULL); dm_get_profile_stages returns all five
 * stage means in ms[0..4] = mask rows, LM head, JS pass 1, JS pass 2, vote/accept (a stage
 * that launched no kernel in a call counts 0 for that call: the JS passes of dropmatch_verify,
 * the vote/accept stage when that step ran inside the LM-head launch; with nucleus sampling
 * ms[2] is the time of all its passes together).  dm_set_profiling(ctx, 2) times only the LM-head contraction
 * kernel, with two events that take the begin and end timestamps of that launch itself (events
 * recorded on the stream around a launch also span the dispatch gap in front of the kernel); the
 * other stage means then read 0.  This is the way to time the dominant kernel inside a timed loop.  dm_set_profiling(ctx, 0) stops recording and forgets
 * the samples.  dm_set_profiling_stride(ctx, n) makes the calls that record events every n-th
 * verify call counted from the next dm_set_profiling (n >= 1, default 1; DM_EINVAL otherwise):
 * an event pair costs a few microseconds of stream time, so a timed loop samples a fraction of
 * its calls.  Recording must be off while a stream is captured into a graph (events cannot be
 * recorded into a capture this way). */
#define DM_PROFILE_MAX_CALLS 512
dm_status dm_set_profiling(dm_ctx* ctx, int32_t enabled);
dm_status dm_set_profiling_stride(dm_ctx* ctx, int32_t stride);
dm_status dm_get_profile(dm_ctx* ctx, int32_t* n_calls, float* ms_mask, float* ms_lmhead, float* ms_vote);
dm_status dm_get_profile_stages(dm_ctx* ctx, int32_t* n_calls, float* ms /* HOST [5] */);
/* The individual durations behind those means: up to n_max samples of stage `stage` (0..4, as above), in
 * the order of the recorded calls, into ms; *n_out = how many (calls in which the stage launched nothing
 * are left out; with dm_set_profiling(ctx, 2) only stage 1 has samples).  Waits for the last recorded event. */
dm_status dm_get_profile_samples(dm_ctx* ctx, int32_t stage, float* ms /* HOST [n_max] */, int32_t n_max, int32_t* n_out);

/* Which contraction kernel a parameter block selects: 0 = generic fp32-FMA tiles (any
 * shape, f32 or bf16), 1 = bf16 MFMA kernel (bf16, d % 64 == 0).  Negative = dm_status. */
int32_t dm_kernel_choice(const dm_params* prm);

#ifdef __cplusplus
}
#endif
#endif /* DROPMATCH_H */
