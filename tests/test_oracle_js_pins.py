"""Pins for the distribution-level part of the CPU oracle (softmax of Eq. (3), centroid of
Eq. (5), the JS rule of Eq. (6), Algorithm 1).  Each check compares the oracle with
something that is not the oracle: hand-derived closed forms (tests/golden), scipy's own
Jensen-Shannon / entropy / softmax routines, exact special cases, and truth tables."""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats
from scipy.spatial.distance import jensenshannon

from oracle import dropmatch_oracle as orc
from paper_2603_03333_amd import workloads as wk

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden():
    out = {}
    with open(os.path.join(GOLDEN, "js_closed_forms.txt")) as f:
        for ln in f:
            if ln.strip() and not ln.startswith("#"):
                k, v = ln.split()
                out[k] = float(v)
    return out


# ---- Jensen-Shannon divergence ------------------------------------------------ #
def test_js_closed_forms():
    g = _golden()
    assert orc.js_divergence([1, 0], [0.5, 0.5]) == pytest.approx(g["three_quarters_ln_4_3"], abs=1e-15)
    assert orc.js_divergence([1, 0], [0, 1]) == pytest.approx(g["ln_2"], abs=1e-15)
    assert orc.js_divergence([0.5, 0.5, 0], [0, 0.5, 0.5]) == pytest.approx(g["half_ln_2"], abs=1e-15)
    # the golden numbers are what the hand derivation says
    assert g["three_quarters_ln_4_3"] == pytest.approx(0.75 * math.log(4 / 3), abs=1e-16)
    assert g["ln_2"] == pytest.approx(math.log(2), abs=1e-16)


def test_js_matches_scipy_distance_and_entropy_form():
    rng = np.random.default_rng(5)
    for V in (2, 3, 17, 1000):
        for _ in range(5):
            P = rng.dirichlet(np.full(V, 0.3))
            Q = rng.dirichlet(np.full(V, 2.0))
            if V > 3:
                P[rng.integers(0, V, size=V // 4)] = 0.0     # exact zeros: 0 log 0 = 0
                P /= P.sum()
            js = orc.js_divergence(P, Q)
            assert js == pytest.approx(jensenshannon(P, Q) ** 2, rel=1e-10, abs=1e-14)   # scipy returns sqrt(JS), base e
            M = 0.5 * (P + Q)
            ent = scipy.stats.entropy(M) - 0.5 * scipy.stats.entropy(P) - 0.5 * scipy.stats.entropy(Q)
            assert js == pytest.approx(ent, rel=1e-9, abs=1e-13)
            assert orc.kl_divergence(P, M) == pytest.approx(float(np.sum(scipy.special.rel_entr(P, M))), rel=1e-12)


def test_js_basic_properties():
    rng = np.random.default_rng(6)
    for _ in range(20):
        P = rng.dirichlet(np.ones(50))
        Q = rng.dirichlet(np.ones(50))
        a, b = orc.js_divergence(P, Q), orc.js_divergence(Q, P)
        assert a == pytest.approx(b, rel=1e-13)                   # symmetric
        assert 0.0 <= a <= math.log(2) + 1e-15                    # bounded by ln 2
        assert orc.js_divergence(P, P) == 0.0                     # zero iff equal
    # not the KL divergence (which is asymmetric and unbounded)
    P, Q = np.array([0.9, 0.1]), np.array([0.1, 0.9])
    assert orc.js_divergence(P, Q) < orc.kl_divergence(P, Q)


# ---- softmax and centroid ------------------------------------------------------- #
def test_softmax_matches_scipy_and_is_shift_invariant():
    rng = np.random.default_rng(7)
    l = rng.normal(size=(4, 300)) * 5
    sm = orc.softmax(l)
    assert np.allclose(sm, scipy.special.softmax(l, axis=-1), rtol=1e-13, atol=0)
    assert np.allclose(sm.sum(-1), 1.0, atol=1e-14)
    assert np.allclose(orc.softmax(l + 1000.0), sm, rtol=1e-10)   # no overflow, same result
    assert np.allclose(orc.softmax([0.0, math.log(3.0)]), [0.25, 0.75], atol=1e-15)


def test_centroid_is_softmax_of_mean_logits_not_mean_of_probabilities():
    # hand case: l1 = (0, 0), l2 = (0, 2 ln 3): mean logits (0, ln 3) -> (1/4, 3/4);
    # the mean of the two softmaxes would be ((1/2 + 1/10)/2, (1/2 + 9/10)/2) = (0.3, 0.7)
    L = np.array([[0.0, 0.0], [0.0, 2 * math.log(3.0)]])
    assert np.allclose(orc.centroid(L), [0.25, 0.75], atol=1e-15)
    assert not np.allclose(orc.centroid(L), [0.3, 0.7], atol=1e-3)
    # K = 1: the centroid is that path's own distribution
    l = np.array([[0.3, -1.0, 2.0]])
    assert np.allclose(orc.centroid(l), orc.softmax(l[0]), atol=1e-16)
    # the mean divides by K (a sum instead of a mean would sharpen the distribution)
    L3 = np.array([[1.0, 0.0], [1.0, 0.0], [1.0, 0.0]])
    assert np.allclose(orc.centroid(L3), orc.softmax([1.0, 0.0]), atol=1e-15)


# ---- Eq. (6) and Algorithm 1 ------------------------------------------------------ #
def test_js_rule_hand_case():
    # two heads (1,0)-ish and (0,1)-ish logits; centroid = uniform
    big = 50.0
    L = np.array([[big, 0.0], [0.0, big]])
    pbar = orc.centroid(L)
    assert np.allclose(pbar, [0.5, 0.5], atol=1e-15)
    hit, jd, jh = orc.js_rule([0.5, 0.5], L)
    g = _golden()
    assert jd == 0.0 and hit                                       # draft at the centroid: always inside
    assert jh[0] == pytest.approx(g["three_quarters_ln_4_3"], abs=1e-12)   # each head is (1,0) vs (1/2,1/2)
    assert jh[1] == pytest.approx(g["three_quarters_ln_4_3"], abs=1e-12)
    # a draft farther from the centroid than every head is rejected: impossible here (heads are extreme),
    # so shrink the heads instead
    L2 = np.array([[0.1, 0.0], [0.0, 0.1]])
    hit2, jd2, jh2 = orc.js_rule([0.9, 0.1], L2)
    assert not hit2 and jd2 > jh2.max()
    # "<=": a draft equal to one of the heads sits exactly on the boundary and is accepted
    hit3, jd3, jh3 = orc.js_rule(orc.softmax(L2[0]), L2)
    assert hit3 and jd3 == pytest.approx(jh3[0], rel=1e-12)


def test_js_rule_uses_max_over_heads_not_mean_or_min():
    L = np.array([[3.0, 0.0, 0.0], [0.0, 0.2, 0.0], [0.0, 0.0, 0.1]])
    pbar = orc.centroid(L)
    jh = np.array([orc.js_divergence(orc.softmax(L[i]), pbar) for i in range(3)])
    # a draft whose divergence lies between the mean and the max of the heads' divergences
    for w in np.linspace(0, 1, 101):
        phat = (1 - w) * pbar + w * orc.softmax(L[0])
        jd = orc.js_divergence(phat, pbar)
        if jh.mean() < jd < jh.max():
            assert orc.js_rule(phat, L)[0]
            break
    else:
        pytest.fail("no probe distribution found")


def test_algorithm1_truth_table():
    # js in {accept, reject} x majority in {match, no match} x draft present or not
    L_tight = np.array([[0.1, 0.0, 0.0], [0.0, 0.1, 0.0]])
    near = orc.centroid(L_tight)                 # JS accepts
    far = np.array([0.98, 0.01, 0.01])           # JS rejects
    assert orc.js_rule(near, L_tight)[0] and not orc.js_rule(far, L_tight)[0]
    ids_match, ids_other = [4, 4, 7], [7, 7, 4]
    for phat, ids, want in [(near, ids_match, True), (near, ids_other, True),
                            (far, ids_match, True), (far, ids_other, False)]:
        assert orc.algorithm1_hit(4, phat, L_tight, ids) is want
    assert orc.algorithm1_hit(-1, near, L_tight, ids_match) is False


def _small_problem(seed, B=2, T=4, K=5, d=24, V=40, p=0.3, bonus=True):
    wl = wk.Workload("js", d=d, V=V, dtype="f32", B=B, T=T, K=K, p=p, bonus=bonus, data_seed=seed)
    W = wk.make_weight(wl, sigma=0.3)
    h = wk.make_hidden(wl)
    seeds = wk.make_seeds(wl, base_seed=seed)
    greedy = orc.greedy_ids(h, W)
    draft = wk.make_draft_ids(wl, greedy)
    clean = np.einsum("vd,btd->btv", W.astype(np.float64), h.astype(np.float64))
    probs = wk.make_draft_probs(wl, clean.astype(np.float32))
    return wl, W, h, seeds, draft, probs


def test_verify_js_against_scipy_from_pinned_logits():
    """The whole JS step recomputed with scipy from the path logits that verify() returns
    (those are pinned by the hand cases and brute force of the token-level tests)."""
    for seed in (11, 12, 13):
        wl, W, h, seeds, draft, probs = _small_problem(seed)
        ref = orc.verify(h, W, draft, seeds, wl.K, wl.p, want_logits=(0, wl.V))
        out = orc.verify_js(h, W, draft, probs, seeds, wl.K, wl.p, rule=orc.RULE_JS_OR_MAJORITY)
        only = orc.verify_js(h, W, draft, probs, seeds, wl.K, wl.p, rule=orc.RULE_JS)
        assert np.array_equal(out["path_ids"], ref["path_ids"])
        L = ref["logits"].reshape(wl.B, wl.T, wl.K, wl.V)
        n_js = n_alg = 0
        for b in range(wl.B):
            want_len, want_only = None, None
            for t in range(wl.T):
                pbar = scipy.special.softmax(L[b, t].mean(axis=0))
                jh = np.array([jensenshannon(scipy.special.softmax(L[b, t, i]), pbar) ** 2 for i in range(wl.K)])
                assert np.allclose(out["js_heads"][b, t], jh, rtol=1e-9, atol=1e-13)
                g = int(draft[b, t])
                if g < 0:
                    assert out["js_draft"][b, t] == -1.0 and out["hit"][b, t] == 0 and only["hit"][b, t] == 0
                    js_ok = maj_ok = False
                else:
                    # scipy first renormalises its arguments; a float32 distribution sums to 1 only
                    # within ~1e-7, hence the looser tolerance on the draft side
                    jd = jensenshannon(probs[b, t].astype(np.float64), pbar) ** 2
                    assert out["js_draft"][b, t] == pytest.approx(jd, rel=1e-6, abs=1e-13)
                    assert out["js_margin"][b, t] == pytest.approx(jh.max() - jd, abs=1e-7)
                    assert abs(jh.max() - jd) > 1e-6, "probe too close to a tie for this pin"
                    js_ok = jd <= jh.max()
                    vals, cnts = np.unique(ref["path_ids"][b, t], return_counts=True)
                    maj_ok = int(vals[np.argmax(cnts)]) == g          # np.unique sorts: first max = smallest id
                    assert bool(out["hit"][b, t]) == (js_ok or maj_ok)
                    assert bool(only["hit"][b, t]) == js_ok
                    n_js += js_ok
                    n_alg += (js_ok or maj_ok)
                if want_len is None and not (js_ok or maj_ok):
                    want_len = t
                if want_only is None and not js_ok:
                    want_only = t
            assert out["accept_len"][b] == (wl.T if want_len is None else want_len)
            assert only["accept_len"][b] == (wl.T if want_only is None else want_only)
            assert np.array_equal(out["accept_mask"][b], (np.arange(wl.T) < out["accept_len"][b]).astype(np.uint8))
        assert n_alg >= n_js


def test_logits_carry_the_inverted_dropout_scale():
    """Softmax is not scale invariant: the 1/(1-p) of Eq. (2) must be inside the logits that
    Eq. (5)/(6) see.  Recompute one position by hand from the masks."""
    wl, W, h, seeds, draft, probs = _small_problem(21, B=1, T=2, K=3, p=0.5)
    out = orc.verify_js(h, W, draft, probs, seeds, wl.K, wl.p)
    keep = orc.keep_masks(int(seeds[0]), 0, wl.T, wl.K, wl.d, wl.p)
    t = 0
    L = np.stack([(W.astype(np.float64) * (h[0, t].astype(np.float64) * keep[t, i] / 0.5)).sum(axis=1)
                  for i in range(wl.K)])
    pbar = scipy.special.softmax(L.mean(axis=0))
    jh = [jensenshannon(scipy.special.softmax(L[i]), pbar) ** 2 for i in range(wl.K)]
    assert np.allclose(out["js_heads"][0, t], jh, rtol=1e-9)
    unscaled = [jensenshannon(scipy.special.softmax(L[i] * 0.5), scipy.special.softmax(L.mean(axis=0) * 0.5)) ** 2
                for i in range(wl.K)]
    assert not np.allclose(out["js_heads"][0, t], unscaled, rtol=1e-3)


def test_p_zero_heads_collapse():
    """p = 0: every mask keeps everything, all heads coincide with the plain LM head, the
    cluster has zero radius, so Eq. (6) rejects every draft that is not the head's own
    distribution and Algorithm 1 reduces to greedy verification."""
    wl, W, h, seeds, draft, probs = _small_problem(31, p=0.0)
    out = orc.verify_js(h, W, draft, probs, seeds, wl.K, 0.0)
    assert np.all(np.abs(out["js_heads"]) < 1e-15)     # zero up to float64 rounding of the mean
    greedy = orc.greedy_ids(h, W)
    want_hit = (draft == greedy) & (draft >= 0)
    assert np.array_equal(out["hit"].astype(bool), want_hit)


def test_k_one_centroid_is_the_single_head():
    wl, W, h, seeds, draft, probs = _small_problem(41, K=1)
    out = orc.verify_js(h, W, draft, probs, seeds, 1, wl.p, rule=orc.RULE_JS)
    assert np.all(out["js_heads"] == 0.0)
    assert not out["hit"].any()          # noisy drafts: positive divergence > 0 = radius


def test_algorithm1_accepts_superset_of_each_rule():
    for seed in (51, 52):
        wl, W, h, seeds, draft, probs = _small_problem(seed, B=3, T=5, bonus=False)
        alg = orc.verify_js(h, W, draft, probs, seeds, wl.K, wl.p, rule=orc.RULE_JS_OR_MAJORITY)
        js = orc.verify_js(h, W, draft, probs, seeds, wl.K, wl.p, rule=orc.RULE_JS)
        maj = orc.verify(h, W, draft, seeds, wl.K, wl.p, rule=orc.RULE_MAJORITY)
        assert np.array_equal(alg["hit"], js["hit"] | maj["hit"])
        assert np.all(alg["accept_len"] >= js["accept_len"]) and np.all(alg["accept_len"] >= maj["accept_len"])
        assert np.array_equal(alg["vote_ids"], maj["vote_ids"]) and np.array_equal(alg["vote_cnt"], maj["vote_cnt"])


def test_float64_comparison_of_eq6():
    # Eq. (6) is decided in float64: a draft distribution equal to a head sits exactly on the
    # boundary (<= accepts), one a hair farther from the centroid is rejected although the two
    # sides agree to float32 resolution
    L = np.array([[0.2, 0.0], [0.0, 0.2]])
    head = orc.softmax(L[0])
    hit, jd, jh = orc.js_rule(head, L)
    assert jd == jh.max() and hit
    phat = head + np.array([1e-12, -1e-12])
    hit, jd, jh = orc.js_rule(phat, L)
    assert jd > jh.max() and np.float32(jd) == np.float32(jh.max()) and not hit


def test_draft_probs_generator_shapes_and_topk():
    wl, W, h, seeds, draft, probs = _small_problem(61)
    assert probs.dtype == np.float32 and probs.shape == (wl.B, wl.T, wl.V)
    assert np.allclose(probs.sum(-1), 1.0, atol=1e-5) and (probs > 0).all()
    clean = np.einsum("vd,btd->btv", W.astype(np.float64), h.astype(np.float64)).astype(np.float32)
    tk = wk.make_draft_probs(wl, clean, topk=7)
    assert ((tk > 0).sum(-1) == 7).all() and np.allclose(tk.sum(-1), 1.0, atol=1e-5)
    out = orc.verify_js(h, W, draft, tk, seeds, wl.K, wl.p)          # zeros in the draft are fine
    assert np.isfinite(out["js_draft"]).all()


def test_clean_last_path_under_the_js_rules():
    wl, W, h, seeds, draft, probs = _small_problem(81, B=2, T=4, K=6)
    for rule in (orc.RULE_JS, orc.RULE_JS_OR_MAJORITY):
        a = orc.verify_js(h, W, draft, probs, seeds, wl.K, wl.p, rule=rule, clean_last_path=True)
        b = orc.verify_js(h, W, draft, probs, seeds, wl.K - 1, wl.p, rule=rule)
        assert np.array_equal(a["path_ids"][:, :, -1], orc.greedy_ids(h, W))
        assert np.array_equal(a["js_heads"][:, :, :-1], b["js_heads"]) and np.all(a["js_heads"][:, :, -1] == 0)
        for k in ("js_draft", "js_margin", "vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len"):
            assert np.array_equal(a[k], b[k]), k
