"""CPU oracle for the DropMatch Monte-Carlo-dropout LM-head verification step.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the HIP
path is checked against.  Only the test-suite, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path never does, and this module
imports nothing from the product package.  Everything here is numpy in float64 and
Python integers; nothing is blocked, fused or reordered beyond what the method
states, so each function can be read against the paper by eye.

What the paper fixes (Methodology, "Multi-Sample LM Head via MC Dropout" and
"Acceptance Criteria"):

  Eq. (1)  m_j^(i) ~ Bernoulli(1 - p_drop), i.i.d. over j = 1..d, one mask per path i
  Eq. (2)  h_t^(i) = h_t * m^(i) / (1 - p_drop)          (inverted-dropout scaling)
  Eq. (3)  l_t^(i) = W h_t^(i)                           (shared LM-head weight W[V,d])
  y_t^(i) = argmax_v l_t^(i)[v]                          (token of path i; softmax is monotone)
  Eq. (4)  naive token matching: accept iff draft token is in {y_t^(i)}
  Eq. (7)  majority rule: accept iff majority({y_t^(i)}) equals the draft token
  Eq. (3)  p_t^(i) = Softmax(l_t^(i))                    (second half of Eq. (3))
  Eq. (5)  centroid  pbar_t = Softmax((1/K) sum_i l_t^(i))   (mean of LOGITS, then softmax)
  Eq. (6)  JS rule: accept iff JS(phat_t || pbar_t) <= max_i JS(p_t^(i) || pbar_t),
           phat_t being the draft model's distribution at that position
  Alg. 1   accept iff Eq. (6) holds, else iff Eq. (7) holds, else reject
  a rejected position rejects every later one; the count of accepted draft
  tokens is the acceptance length (Metrics paragraph, "Mean Acceptance Length").

What the paper leaves open and this oracle decides (each decision is a reading,
listed with its reason in the design notes of the repository):

  * the random source: Philox4x32-10 (Salmon et al., SC'11), counter
    (j >> 2, t, i, step), key = the sequence's 64-bit seed (low word, high word);
    dimension j takes output word j & 3; keep iff word >= floor(p * 2^32),
    p being the float32 the caller passes, widened exactly to float64;
  * a fresh mask per (path, position) unless `share_mask_across_pos` (then t := 0);
  * argmax ties -> smallest vocabulary index;  majority = plurality (mode) of the K
    tokens (the paper's agreement table lists majority sizes 1..5 for K = 5),
    ties between modes -> smallest token id;
  * draft id < 0 means "no draft token at this row" and never matches;
  * sampled path tokens (the paper says a path's token may be "selected by nucleus sampling"
    instead of the arg max, without parameters): with a temperature tau the token of path i
    is drawn from Softmax(l^(i) / tau) by the Gumbel-max construction,
    y = argmax_v (l[v] / tau + g[v]), g[v] = -ln(-ln u[v]), with u[v] = ((w >> 9) + 1/2) 2^-23
    and w the Philox4x32-10 word (v & 3) of counter (v >> 2, t, i, step) under the key
    seed + 0x9E3779B97F4A7C15 (mod 2^64) - a stream separate from the masks'.  With top_p < 1
    the draw is restricted to the nucleus of Softmax(l / tau): most probable tokens first until
    their probabilities add up to top_p, tokens exactly as probable as the last one included
    (so the set does not depend on an order among equals); same noise, arg max over the set;
  * `clean_last_path` (the paper does not say which token is emitted after a rejection
    or as the bonus token): path K-1 of every row is the plain LM head, h_t itself
    with no mask and no scale; its token is reported in path_ids[..., K-1] and the
    rules (Eq. (4), (6), (7), Alg. 1) use paths 0..K-2 only;
  * Jensen-Shannon divergence (the paper names it without a formula): the standard
    JS(P||Q) = KL(P||M)/2 + KL(Q||M)/2 with M = (P+Q)/2, natural logarithm,
    0 log 0 = 0; the two sides of Eq. (6) are compared in float64 (a test that compares
    a float32 implementation with this owns the band around a tie);
  * the JS rule and Alg. 1 are defined for chains only (the paper uses tree
    decoding only together with naive token matching);
  * tree verification: parent[n] < n, node 0 is the root (always accepted); node n
    is accepted iff its parent is accepted and the rule holds for draft[n] against
    the K path tokens of row parent[n]; result = depth of the deepest accepted node.

Pins (tests/test_oracle_*.py, all CPU): Philox known-answer vectors and an
independent big-integer implementation; exact integer thresholds by rational
arithmetic; keep-rate and E[h^(i)] = h statistics; p = 0 reducing to plain greedy
verification through a separate library matmul; hand-checkable integer cases by
brute force in exact rational arithmetic; identical masks -> identical paths;
rule set-relations; chain/tree equivalence; batch independence.
JS part: JS against scipy's Jensen-Shannon distance and entropy routines, the
closed form 3/4 ln(4/3), disjoint/identical supports, the centroid against a hand
case where the mean of logits and the mean of probabilities differ, Alg. 1's
truth table, K = 1 and p = 0 special cases, and the whole JS step against a
separate scipy computation from the (separately pinned) path logits.
Parity unpinned: nothing in this file.  (Task quality on real text - accuracy,
acceptance length on benchmarks - is not computed here at all.)
"""
from __future__ import annotations

import numpy as np

RULE_ANY = 0       # Eq. (4): draft token is one of the K path tokens
RULE_MAJORITY = 1  # Eq. (7): draft token is the most frequent path token
RULE_JS = 2           # Eq. (6) alone: draft distribution within the cluster of head distributions
RULE_JS_OR_MAJORITY = 3  # Algorithm 1: Eq. (6), else Eq. (7)

_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_LO32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


# --------------------------------------------------------------------------- #
# Random source (reading of Eq. (1): the paper only says "i.i.d. Bernoulli")
# --------------------------------------------------------------------------- #
def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
    numbers: as easy as 1, 2, 3", SC'11).  All arguments broadcast; each holds
    32-bit words.  Returns four uint32 arrays.

    One round maps (c0,c1,c2,c3) to (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1,
    lo(M0*c0)); the key is bumped by the Weyl constants between rounds.
    """
    c0, c1, c2, c3, k0, k1 = np.broadcast_arrays(
        *(np.asarray(x, dtype=np.uint64) & _LO32 for x in (c0, c1, c2, c3, k0, k1)))
    for r in range(10):
        p0 = _PHILOX_M0 * c0          # < 2^64, exact in uint64
        p1 = _PHILOX_M1 * c2
        kk0 = (k0 + np.uint64((_PHILOX_W0 * r) & 0xFFFFFFFF)) & _LO32
        kk1 = (k1 + np.uint64((_PHILOX_W1 * r) & 0xFFFFFFFF)) & _LO32
        n0 = (p1 >> _SH32) ^ c1 ^ kk0
        n1 = p1 & _LO32
        n2 = (p0 >> _SH32) ^ c3 ^ kk1
        n3 = p0 & _LO32
        c0, c1, c2, c3 = n0, n1, n2, n3
    return tuple(x.astype(np.uint32) for x in (c0, c1, c2, c3))


def drop_threshold(p) -> int:
    """Integer t such that a uniform 32-bit word u is DROPPED iff u < t.

    t = floor(p * 2^32) with p the float32 value widened to float64 (exact: a
    float32 times 2^32 is representable).  P(keep) = 1 - t / 2^32.
    """
    p64 = float(np.float32(p))
    if not (0.0 <= p64 < 1.0):
        raise ValueError("p_drop must satisfy 0 <= p < 1")
    return int(np.floor(p64 * 4294967296.0))


def keep_mask(seed: int, step: int, t: int, i: int, d: int, p) -> np.ndarray:
    """Eq. (1): keep-mask m^(i) in {0,1}^d of path i at row t, as bool[d]."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    nctr = (d + 3) // 4                      # counter c serves dimensions 4c .. 4c+3
    words = philox4x32_10(np.arange(nctr, dtype=np.uint64), t, i, step,
                          seed & 0xFFFFFFFF, seed >> 32)
    u = np.stack(words, axis=1).reshape(-1)[:d]          # u[j] = word (j & 3) of counter j >> 2
    return u.astype(np.uint64) >= np.uint64(drop_threshold(p))


def keep_masks(seed: int, step: int, T: int, K: int, d: int, p,
               share_mask_across_pos: bool = False) -> np.ndarray:
    """All masks of one sequence, bool[T, K, d].  With `share_mask_across_pos`
    path i uses one mask at every row (position word of the counter forced to 0)."""
    out = np.empty((T, K, d), dtype=bool)
    for t in range(T):
        for i in range(K):
            out[t, i] = keep_mask(seed, step, 0 if share_mask_across_pos else t, i, d, p)
    return out


def pack_mask_bits(keep: np.ndarray) -> np.ndarray:
    """Bit-pack bool[..., d] to uint32[..., ceil(d/32)]: word w holds dimensions
    32w .. 32w+31, bit (j & 31) is keep(j); bits past d are zero."""
    d = keep.shape[-1]
    nw = (d + 31) // 32
    padded = np.zeros(keep.shape[:-1] + (nw * 32,), dtype=np.uint64)
    padded[..., :d] = keep
    weights = np.uint64(1) << np.arange(32, dtype=np.uint64)
    return (padded.reshape(keep.shape[:-1] + (nw, 32)) * weights).sum(axis=-1).astype(np.uint32)


# --------------------------------------------------------------------------- #
# Eq. (2), Eq. (3), path token
# --------------------------------------------------------------------------- #
def masked_state(h_t: np.ndarray, keep: np.ndarray, p) -> np.ndarray:
    """Eq. (2): h_t^(i) = h_t * m^(i) / (1 - p_drop), float64."""
    p64 = float(np.float32(p))
    return np.asarray(h_t, dtype=np.float64) * keep.astype(np.float64) / (1.0 - p64)


def path_logits(W: np.ndarray, h_t: np.ndarray, keep: np.ndarray, p) -> np.ndarray:
    """Eq. (3): l_t^(i) = W h_t^(i), float64[V]."""
    return np.asarray(W, dtype=np.float64) @ masked_state(h_t, keep, p)


def path_token(logits: np.ndarray):
    """y = argmax_v l[v], ties -> smallest v.  Also returns top1 - top2 (inf if V == 1)."""
    y = int(np.argmax(logits))            # numpy returns the first maximal index
    if logits.shape[0] < 2:
        return y, float("inf")
    top2 = np.partition(logits, -2)[-2:]
    return y, float(top2[1] - top2[0])


def tokens_within(values: np.ndarray, tol: float):
    """Test support, not a step of the method: every index whose value is within `tol` of the
    maximum, ascending, with its distance from the maximum.  These are the tokens a float32
    implementation may legitimately return for a row whose top-1 is not clear of its rounding
    errors; the parity tests accept exactly these and nothing else."""
    values = np.asarray(values, dtype=np.float64)
    deficit = np.max(values) - values
    ids = np.nonzero(deficit <= float(tol))[0]
    return ids.astype(np.int64), deficit[ids]


def row_states(h_t, seed, step, tt, K, d, p, clean_last_path=False):
    """The K inputs of the LM head for one row, [K, d]: Eq. (1)-(2) for every path, except that
    with `clean_last_path` the last one is h_t itself (no mask, no scale)."""
    rows = [masked_state(h_t, keep_mask(seed, step, tt, i, d, p), p) for i in range(K)]
    if clean_last_path:
        if K < 2:
            raise ValueError("clean_last_path needs K >= 2")
        rows[K - 1] = np.asarray(h_t, dtype=np.float64).copy()
    return np.stack(rows, axis=0)


SAMPLE_KEY_OFFSET = 0x9E3779B97F4A7C15    # added to the sequence seed for the sampling stream


def sampling_uniforms(seed: int, step: int, t: int, i: int, V: int) -> np.ndarray:
    """u[v] in (0, 1) for the sampled token of path i at row t: 23 random bits per vocabulary
    entry, centred in their cell so that u is exact in float32 and never 0 or 1."""
    key = (int(seed) + SAMPLE_KEY_OFFSET) & 0xFFFFFFFFFFFFFFFF
    nctr = (V + 3) // 4
    words = philox4x32_10(np.arange(nctr, dtype=np.uint64), t, i, step, key & 0xFFFFFFFF, key >> 32)
    w = np.stack(words, axis=1).reshape(-1)[:V].astype(np.uint64)
    return ((w >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def gumbel_noise(u: np.ndarray) -> np.ndarray:
    """Standard Gumbel variates g = -ln(-ln u) (quantile function of the Gumbel distribution)."""
    u = np.asarray(u, dtype=np.float64)
    return -np.log(-np.log1p(-(1.0 - u)))      # ln u through log1p: exact near u = 1, where g is largest


def nucleus(z: np.ndarray, top_p: float):
    """The nucleus (top-p set, Holtzman et al. 2020, the sampling the paper names for path tokens)
    of Softmax(z): the tokens in order of decreasing probability (equal ones: smaller id first)
    up to and including the first at which the running sum reaches top_p; tokens exactly as
    probable as the last one taken are all in, so that the set does not depend on how equal
    tokens are ordered.  Returns (boolean mask over the vocabulary, number n of tokens taken
    before the ties were added)."""
    q = softmax(np.asarray(z, dtype=np.float64))
    order = np.argsort(-q, kind="stable")
    cum = np.cumsum(q[order])
    n = min(int(np.searchsorted(cum, float(top_p), side="left")) + 1, q.size)
    return q >= q[order[n - 1]], n


def sampled_values(logits: np.ndarray, tau: float, g: np.ndarray, top_p=None) -> np.ndarray:
    """The perturbed values logits[v] / tau + g[v] whose arg max is the Gumbel-max draw from
    Softmax(logits / tau); with top_p, -inf outside the nucleus of that distribution."""
    z = np.asarray(logits, dtype=np.float64) / float(tau)
    y = z + g
    if top_p is not None:
        y = np.where(nucleus(z, top_p)[0], y, -np.inf)
    return y


def sampled_token(logits: np.ndarray, tau: float, g: np.ndarray, top_p=None):
    """Gumbel-max draw from Softmax(logits / tau): argmax_v (logits[v] / tau + g[v]), ties ->
    smallest v.  With top_p the arg max runs over the nucleus of that distribution only, which
    is a draw from the distribution renormalised on the nucleus (the noise of the other tokens
    is simply not looked at).  Also returns the top-1 minus top-2 gap of the perturbed values
    (inf when a single token is eligible)."""
    tok, gap = path_token(sampled_values(logits, tau, g, top_p))
    return tok, (gap if np.isfinite(gap) else np.inf)


# --------------------------------------------------------------------------- #
# Eq. (4), Eq. (7), prefix / tree acceptance
# --------------------------------------------------------------------------- #
def vote(ids):
    """Mode of the K path tokens (Eq. (7), "majority"): returns (token, count);
    among equally frequent tokens the smallest id wins."""
    counts = {}
    for y in ids:
        counts[int(y)] = counts.get(int(y), 0) + 1
    best = max(counts.values())
    return min(tok for tok, c in counts.items() if c == best), best


def rule_hit(draft: int, ids, rule: int) -> bool:
    """Acceptance test of one draft token against the K path tokens of one row."""
    draft = int(draft)
    if draft < 0:
        return False
    if rule == RULE_ANY:                       # Eq. (4)
        return any(int(y) == draft for y in ids)
    if rule == RULE_MAJORITY:                  # Eq. (7)
        return vote(ids)[0] == draft
    raise ValueError("unknown rule")


def accept_chain(hit):
    """Prefix rule: the first rejected row rejects all later ones.
    Returns (accept_len, best_node, accept_mask)."""
    T = len(hit)
    mask = np.zeros(T, dtype=np.uint8)
    n = 0
    while n < T and hit[n]:
        mask[n] = 1
        n += 1
    return n, n - 1, mask


def accept_tree(edge_hit, parent):
    """Tree of draft candidates in topological order (parent[n] < n, parent[0] = -1).
    Node 0 is accepted; node n > 0 is accepted iff its parent is and edge_hit[n].
    Returns (max accepted depth, that node - smallest index on ties, accept_mask)."""
    T = len(parent)
    acc = np.zeros(T, dtype=np.uint8)
    depth = np.zeros(T, dtype=np.int64)
    acc[0] = 1
    best_depth, best = 0, 0
    for n in range(1, T):
        q = int(parent[n])
        if not (0 <= q < n):
            raise ValueError("parent[] is not a topological order rooted at node 0")
        depth[n] = depth[q] + 1
        acc[n] = 1 if (acc[q] and edge_hit[n]) else 0
        if acc[n] and depth[n] > best_depth:
            best_depth, best = int(depth[n]), n
    return best_depth, best, acc


# --------------------------------------------------------------------------- #
# Eq. (3) softmax, Eq. (5) centroid, Eq. (6) JS rule, Algorithm 1
# --------------------------------------------------------------------------- #
def softmax(l: np.ndarray) -> np.ndarray:
    """Softmax over the last axis, float64 (second half of Eq. (3))."""
    l = np.asarray(l, dtype=np.float64)
    e = np.exp(l - np.max(l, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def centroid(L: np.ndarray) -> np.ndarray:
    """Eq. (5): pbar = Softmax of the MEAN over the K paths of their logits.  L is [K, V]."""
    L = np.asarray(L, dtype=np.float64)
    return softmax(np.sum(L, axis=0) / L.shape[0])


def kl_divergence(P: np.ndarray, Q: np.ndarray) -> float:
    """KL(P || Q) = sum_v P[v] ln(P[v] / Q[v]), terms with P[v] = 0 contribute 0."""
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    nz = P > 0
    return float(np.sum(P[nz] * (np.log(P[nz]) - np.log(Q[nz]))))


def js_divergence(P: np.ndarray, Q: np.ndarray) -> float:
    """Jensen-Shannon divergence JS(P || Q) = KL(P || M)/2 + KL(Q || M)/2, M = (P + Q)/2."""
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    M = 0.5 * (P + Q)
    return 0.5 * kl_divergence(P, M) + 0.5 * kl_divergence(Q, M)


def js_rule(p_hat: np.ndarray, L: np.ndarray):
    """Eq. (6) for one position.  p_hat[V]: draft distribution; L[K, V]: path logits.
    Returns (hit, js_draft, js_heads[K]).  The comparison is made in float64."""
    pbar = centroid(L)
    js_heads = np.array([js_divergence(softmax(L[i]), pbar) for i in range(L.shape[0])])
    js_draft = js_divergence(np.asarray(p_hat, dtype=np.float64), pbar)
    hit = bool(js_draft <= np.max(js_heads))
    return hit, js_draft, js_heads


def algorithm1_hit(draft: int, p_hat: np.ndarray, L: np.ndarray, ids) -> bool:
    """Algorithm 1 for one position: accept by Eq. (6); otherwise accept by Eq. (7);
    otherwise reject.  (A row without a draft token never hits.)"""
    if int(draft) < 0:
        return False
    if js_rule(p_hat, L)[0]:
        return True
    return rule_hit(draft, ids, RULE_MAJORITY)


def verify_js(h, W, draft_ids, draft_probs, seeds, K: int, p, step: int = 0,
              rule: int = RULE_JS_OR_MAJORITY, share_mask_across_pos: bool = False,
              clean_last_path: bool = False, near_tol: float = 1e-2):
    """One verification step with the distribution-level rule (chains only).

    draft_probs [B, T, V]: the draft model's distribution for the token row t verifies
    (ignored at rows whose draft id is < 0).  rule: RULE_JS (Eq. (6) alone) or
    RULE_JS_OR_MAJORITY (Algorithm 1).

    Returns what verify() returns plus js_draft[B,T] (-1 at rows without a draft
    token), js_heads[B,T,K] (0 in the slot of a clean last path), and js_margin[B,T] =
    max_i js_heads - js_draft (the
    distance of the Eq. (6) decision from a tie; +inf at rows without a draft token), and
    `near` as verify() does.
    """
    if rule not in (RULE_JS, RULE_JS_OR_MAJORITY):
        raise ValueError("verify_js takes RULE_JS or RULE_JS_OR_MAJORITY")
    h = np.asarray(h, dtype=np.float64)
    W64 = np.asarray(W, dtype=np.float64)
    draft_ids = np.asarray(draft_ids)
    B, T, d = h.shape
    V = W64.shape[0]
    draft_probs = np.asarray(draft_probs)
    if W64.shape[1] != d or draft_ids.shape != (B, T) or draft_probs.shape != (B, T, V) or len(seeds) != B:
        raise ValueError("shape mismatch")

    KU = K - 1 if clean_last_path else K      # paths the rules use
    path_ids = np.zeros((B, T, K), dtype=np.int32)
    gap = np.zeros((B, T, K), dtype=np.float64)
    js_draft = np.full((B, T), -1.0)
    js_heads = np.zeros((B, T, K))
    js_margin = np.full((B, T), np.inf)
    hit = np.zeros((B, T), dtype=np.uint8)
    near = {}
    for b in range(B):
        for t in range(T):
            tt = 0 if share_mask_across_pos else t
            Hm = row_states(h[b, t], seeds[b], step, tt, K, d, p, clean_last_path)   # Eq. (1)-(2), [K, d]
            L = (W64 @ Hm.T).T                                   # Eq. (3), [K, V]
            for i in range(K):
                path_ids[b, t, i], gap[b, t, i] = path_token(L[i])
                if gap[b, t, i] <= near_tol:
                    near[(b, t, i)] = tokens_within(L[i], near_tol)
            g = int(draft_ids[b, t])
            js_hit, jd, jh = js_rule(draft_probs[b, t], L[:KU])
            js_heads[b, t, :KU] = jh
            if g < 0:
                continue
            js_draft[b, t] = jd
            js_margin[b, t] = float(np.max(jh)) - jd
            if rule == RULE_JS:
                hit[b, t] = js_hit
            else:
                hit[b, t] = js_hit or rule_hit(g, path_ids[b, t, :KU], RULE_MAJORITY)

    out = acceptance_from_hits(hit)
    votes = acceptance_from_path_ids(path_ids[:, :, :KU], draft_ids, RULE_MAJORITY)
    out.update(vote_ids=votes["vote_ids"], vote_cnt=votes["vote_cnt"], path_ids=path_ids, gap=gap,
               js_draft=js_draft, js_heads=js_heads, js_margin=js_margin, near=near, near_tol=float(near_tol))
    return out


def acceptance_from_hits(hit):
    """Prefix rule applied to given per-row decisions hit[B, T] (chain)."""
    hit = np.asarray(hit, dtype=np.uint8)
    B, T = hit.shape
    accept_mask = np.zeros((B, T), dtype=np.uint8)
    accept_len = np.zeros(B, dtype=np.int32)
    best_node = np.zeros(B, dtype=np.int32)
    for b in range(B):
        accept_len[b], best_node[b], accept_mask[b] = accept_chain(hit[b])
    return dict(hit=hit, accept_mask=accept_mask, accept_len=accept_len, best_node=best_node)


# --------------------------------------------------------------------------- #
# The whole step
# --------------------------------------------------------------------------- #
def verify(h, W, draft_ids, seeds, K: int, p, step: int = 0, rule: int = RULE_ANY,
           share_mask_across_pos: bool = False, parent=None, want_logits=None,
           clean_last_path: bool = False, temperature=None, top_p=None, near_tol: float = 1e-2):
    """One DropMatch verification step for B sequences.

    h          [B, T, d]  final hidden states (any float dtype; used as float64)
    W          [V, d]     LM-head weight
    draft_ids  [B, T]     chain: token verified by row t;  tree: token of node t
    seeds      [B]        64-bit mask seed per sequence
    parent     None (chain) or [B, T] (tree)
    want_logits optional (v0, v1): also return logits[B*T*K, v1-v0] for parity of values
    temperature None: path token = arg max.  A positive number: path token sampled from
               Softmax(l / temperature) (see sampled_token; a clean last path stays arg max);
               `gap` then refers to the perturbed values
    top_p      with a temperature: sample from the nucleus of that distribution only (see nucleus)
    near_tol   test support: for every row whose gap is at most near_tol, `near[(b, t, i)]` lists the
               tokens whose (perturbed) value is within near_tol of the row's maximum, with their
               distances from it (see tokens_within)

    Returns a dict of numpy arrays: path_ids[B,T,K], gap[B,T,K] (top-1 minus top-2
    logit of each path), vote_ids[B,T], vote_cnt[B,T], hit[B,T], accept_mask[B,T],
    accept_len[B], best_node[B], near, near_tol (and logits if asked).
    """
    h = np.asarray(h, dtype=np.float64)
    W64 = np.asarray(W, dtype=np.float64)
    draft_ids = np.asarray(draft_ids)
    B, T, d = h.shape
    V = W64.shape[0]
    if W64.shape[1] != d or draft_ids.shape != (B, T) or len(seeds) != B or K < 1:
        raise ValueError("shape mismatch")

    path_ids = np.zeros((B, T, K), dtype=np.int32)
    gap = np.zeros((B, T, K), dtype=np.float64)
    near = {}
    logits_out = None
    if want_logits is not None:
        v0, v1 = want_logits
        logits_out = np.zeros((B * T * K, v1 - v0), dtype=np.float64)

    for b in range(B):
        for t in range(T):
            tt = 0 if share_mask_across_pos else t
            # K masked states of this row, Eq. (1)-(2)
            Hm = row_states(h[b, t], seeds[b], step, tt, K, d, p, clean_last_path)   # [K, d]
            L = W64 @ Hm.T                                       # Eq. (3), [V, K]
            for i in range(K):
                if temperature is None or (clean_last_path and i == K - 1):
                    values = L[:, i]
                    path_ids[b, t, i], gap[b, t, i] = path_token(values)
                else:
                    g = gumbel_noise(sampling_uniforms(seeds[b], step, t, i, V))
                    values = sampled_values(L[:, i], temperature, g, top_p)
                    path_ids[b, t, i], gap[b, t, i] = sampled_token(L[:, i], temperature, g, top_p)
                if gap[b, t, i] <= near_tol:
                    near[(b, t, i)] = tokens_within(values, near_tol)
                if logits_out is not None:
                    logits_out[(b * T + t) * K + i] = L[v0:v1, i]

    KU = K - 1 if clean_last_path else K      # paths the rules use
    out = acceptance_from_path_ids(path_ids[:, :, :KU], draft_ids, rule, parent)
    out["path_ids"] = path_ids
    out["gap"] = gap
    out["near"] = near
    out["near_tol"] = float(near_tol)
    if logits_out is not None:
        out["logits"] = logits_out
    return out


def acceptance_from_path_ids(path_ids, draft_ids, rule: int = RULE_ANY, parent=None):
    """Eq. (4)/(7) and the prefix (or tree) rule applied to given path tokens.
    Split out so that acceptance can also be re-derived from another set of path
    tokens (used when a near-tie legitimately flips a path token)."""
    path_ids = np.asarray(path_ids)
    draft_ids = np.asarray(draft_ids)
    B, T, K = path_ids.shape
    vote_ids = np.zeros((B, T), dtype=np.int32)
    vote_cnt = np.zeros((B, T), dtype=np.int32)
    hit = np.zeros((B, T), dtype=np.uint8)
    accept_mask = np.zeros((B, T), dtype=np.uint8)
    accept_len = np.zeros(B, dtype=np.int32)
    best_node = np.zeros(B, dtype=np.int32)
    for b in range(B):
        for t in range(T):
            vote_ids[b, t], vote_cnt[b, t] = vote(path_ids[b, t])
        if parent is None:
            for t in range(T):
                hit[b, t] = rule_hit(draft_ids[b, t], path_ids[b, t], rule)
            accept_len[b], best_node[b], accept_mask[b] = accept_chain(hit[b])
        else:
            par = np.asarray(parent)[b]
            hit[b, 0] = 1
            for n in range(1, T):
                hit[b, n] = rule_hit(draft_ids[b, n], path_ids[b, int(par[n])], rule)
            accept_len[b], best_node[b], accept_mask[b] = accept_tree(hit[b], par)
    return dict(vote_ids=vote_ids, vote_cnt=vote_cnt, hit=hit, accept_mask=accept_mask,
                accept_len=accept_len, best_node=best_node)


def greedy_ids(h, W):
    """Plain LM head without dropout: argmax_v (W h_t)[v] per row, int32[B, T].
    (The p = 0 special case of the step; also used to plant draft tokens.)"""
    h = np.asarray(h, dtype=np.float64)
    W64 = np.asarray(W, dtype=np.float64)
    B, T, d = h.shape
    out = np.zeros((B, T), dtype=np.int32)
    for b in range(B):
        for t in range(T):
            out[b, t] = path_token(W64 @ h[b, t])[0]
    return out
