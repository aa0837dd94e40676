"""Pins for the sampled path tokens of the CPU oracle (the paper's remark that a path's token may be
chosen by sampling instead of the arg max): the uniforms, the Gumbel transform against scipy's
quantile function, the Gumbel-max theorem by a chi-square test against the softmax it must sample
from, and limits (temperature -> 0 gives the arg max, a large one the uniform distribution)."""
import numpy as np
import scipy.special
import scipy.stats

from oracle import dropmatch_oracle as orc
from paper_2603_03333_amd import workloads as wk
from test_oracle_pins import philox_int


def test_uniforms_are_on_the_23_bit_grid_and_use_their_own_stream():
    seed, step, t, i, V = 12345678901234567, 3, 2, 4, 50
    u = orc.sampling_uniforms(seed, step, t, i, V)
    key = (seed + 0x9E3779B97F4A7C15) & (2 ** 64 - 1)
    for v in (0, 1, 2, 3, 4, 17, 49):
        w = philox_int((v >> 2, t, i, step), (key & 0xFFFFFFFF, key >> 32))[v & 3]
        assert u[v] == ((w >> 9) + 0.5) / 2 ** 23
    assert (u > 0).all() and (u < 1).all()
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)        # exact in float32
    # not the words the masks use (key without the offset)
    wm = philox_int((0, t, i, step), (seed & 0xFFFFFFFF, seed >> 32))[0]
    assert u[0] != ((wm >> 9) + 0.5) / 2 ** 23
    # every component of the key changes the draw
    base = orc.sampling_uniforms(1, 0, 0, 0, 64)
    for other in (orc.sampling_uniforms(2, 0, 0, 0, 64), orc.sampling_uniforms(1, 1, 0, 0, 64),
                  orc.sampling_uniforms(1, 0, 1, 0, 64), orc.sampling_uniforms(1, 0, 0, 1, 64)):
        assert (other != base).mean() > 0.9


def test_gumbel_transform_is_the_gumbel_quantile_function():
    u = np.unique(np.concatenate([(np.arange(0, 2 ** 23, 99991) + 0.5) / 2 ** 23, [0.5 / 2 ** 23, 1 - 0.5 / 2 ** 23]]))
    g = orc.gumbel_noise(u)
    assert np.allclose(g, scipy.stats.gumbel_r.ppf(u), rtol=1e-9, atol=1e-9)
    assert np.all(np.diff(g) > 0)
    assert orc.gumbel_noise(np.exp(-1.0)) == 0.0 or abs(orc.gumbel_noise(np.exp(-1.0))) < 1e-15   # -ln(-ln e^-1) = 0
    # the largest value a 23-bit uniform can give: -ln(-ln(1 - 2^-24)) = 24 ln 2 up to 3e-8
    assert abs(g[-1] - 24 * np.log(2.0)) < 1e-7


def test_gumbel_max_samples_the_softmax():
    rng = np.random.default_rng(3)
    logits = rng.normal(size=7) * 1.5
    for tau in (0.7, 1.0, 2.5):
        want = scipy.special.softmax(logits / tau)
        counts = np.zeros(7)
        n = 10000
        for step in range(n):
            g = orc.gumbel_noise(orc.sampling_uniforms(99, step, 1, 2, 7))
            counts[orc.sampled_token(logits, tau, g)[0]] += 1
        chi2, pval = scipy.stats.chisquare(counts, want * n)
        assert pval > 1e-3, (tau, counts, want * n)
        # and not the distribution at another temperature
        other = scipy.special.softmax(logits / (tau * 2))
        assert scipy.stats.chisquare(counts, other * n)[1] < 1e-6


def test_temperature_limits():
    logits = np.array([0.3, 2.0, -1.0, 1.9])
    g = orc.gumbel_noise(orc.sampling_uniforms(5, 0, 0, 0, 4))
    assert orc.sampled_token(logits, 1e-4, g)[0] == 1          # tau -> 0: the arg max
    counts = np.zeros(4)
    for step in range(4000):
        counts[orc.sampled_token(logits, 1e6, orc.gumbel_noise(orc.sampling_uniforms(5, step, 0, 0, 4)))[0]] += 1
    assert scipy.stats.chisquare(counts)[1] > 1e-3             # tau -> inf: uniform


def test_verify_with_sampled_paths():
    wl = wk.Workload("samp", d=32, V=50, dtype="f32", B=2, T=4, K=6, p=0.2, bonus=True, data_seed=91)
    W, h, seeds = wk.make_weight(wl, sigma=0.3), wk.make_hidden(wl), wk.make_seeds(wl, base_seed=8)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    tau = 0.8
    out = orc.verify(h, W, draft, seeds, wl.K, wl.p, temperature=tau, want_logits=(0, wl.V))
    L = out["logits"].reshape(wl.B, wl.T, wl.K, wl.V)
    for b in range(wl.B):
        for t in range(wl.T):
            for i in range(wl.K):
                g = scipy.stats.gumbel_r.ppf(orc.sampling_uniforms(seeds[b], 0, t, i, wl.V))
                assert out["path_ids"][b, t, i] == int(np.argmax(L[b, t, i] / tau + g))
    # rules act on the sampled tokens
    exp = orc.acceptance_from_path_ids(out["path_ids"], draft, orc.RULE_ANY)
    assert np.array_equal(out["hit"], exp["hit"]) and np.array_equal(out["accept_len"], exp["accept_len"])
    # a clean last path stays the greedy token; the other paths are those of the K-1 run
    c = orc.verify(h, W, draft, seeds, wl.K, wl.p, temperature=tau, clean_last_path=True)
    assert np.array_equal(c["path_ids"][:, :, -1], orc.greedy_ids(h, W))
    assert np.array_equal(c["path_ids"][:, :, :-1], orc.verify(h, W, draft, seeds, wl.K - 1, wl.p, temperature=tau)["path_ids"])
    # sampling differs from the arg max somewhere, and a tiny temperature brings the arg max back
    plain = orc.verify(h, W, draft, seeds, wl.K, wl.p)
    assert (out["path_ids"] != plain["path_ids"]).any()
    assert np.array_equal(orc.verify(h, W, draft, seeds, wl.K, wl.p, temperature=1e-5)["path_ids"], plain["path_ids"])


# ------------------------------------------------------------------ nucleus (top-p) truncation
def test_nucleus_hand_cases():
    q = np.array([0.05, 0.5, 0.15, 0.3])
    z = np.log(q)
    for top_p, members in ((0.4, [1]), (0.51, [1, 3]), (0.79, [1, 3]), (0.81, [1, 2, 3]), (0.94, [1, 2, 3]),
                           (0.96, [0, 1, 2, 3]), (1.0, [0, 1, 2, 3])):
        mask, n = orc.nucleus(z, top_p)
        assert np.flatnonzero(mask).tolist() == members and n == len(members), top_p
    # tokens exactly as probable as the last one taken are all in: 0.4 + 0.2 reaches 0.5 with two
    # tokens, the other two 0.2s come along
    mask, n = orc.nucleus(np.log(np.array([0.2, 0.4, 0.2, 0.2])), 0.5)
    assert n == 2 and mask.all()
    # a shift of the logits changes nothing
    assert np.array_equal(orc.nucleus(z + 123.0, 0.81)[0], orc.nucleus(z, 0.81)[0])


def test_nucleus_is_the_smallest_heaviest_set():
    """Brute force over all subsets of a small vocabulary: among the subsets whose probability
    reaches top_p, the nucleus has the fewest tokens, and among those of that size the most mass."""
    import itertools
    rng = np.random.default_rng(12)
    for trial in range(20):
        V = int(rng.integers(2, 9))
        z = rng.normal(size=V) * 2.0
        q = scipy.special.softmax(z)
        top_p = float(rng.uniform(0.05, 0.999))
        mask, n = orc.nucleus(z, top_p)
        best = None
        for size in range(1, V + 1):
            ok = [(q[list(c)].sum(), c) for c in itertools.combinations(range(V), size) if q[list(c)].sum() >= top_p]
            if ok:
                best = max(ok)[1]
                break
        assert mask.sum() == n == len(best) and set(np.flatnonzero(mask)) == set(best)


def test_nucleus_sets_are_nested_and_limits():
    rng = np.random.default_rng(4)
    z = rng.normal(size=200) * 3.0
    prev = np.zeros(200, dtype=bool)
    for top_p in (1e-9, 0.1, 0.3, 0.5, 0.9, 0.99, 0.999999, 1.0):
        mask, n = orc.nucleus(z, top_p)
        assert (mask | prev).sum() == mask.sum()          # the earlier set is inside
        assert scipy.special.softmax(z)[mask].sum() >= min(top_p, 1.0) - 1e-12
        prev = mask
    assert orc.nucleus(z, 1e-9)[0].sum() == 1 and orc.nucleus(z, 1.0)[0].all()
    g = orc.gumbel_noise(orc.sampling_uniforms(3, 0, 0, 0, 200))
    # top_p -> 0: the arg max whatever the noise; top_p = 1: the unrestricted draw
    assert orc.sampled_token(z, 1.0, g, 1e-9) == (int(np.argmax(z)), np.inf)
    assert orc.sampled_token(z, 0.7, g, 1.0)[0] == orc.sampled_token(z, 0.7, g)[0]


def test_nucleus_draws_follow_the_renormalised_distribution():
    rng = np.random.default_rng(8)
    logits = rng.normal(size=9) * 1.5
    tau, top_p = 0.9, 0.8
    q = scipy.special.softmax(logits / tau)
    mask, _ = orc.nucleus(logits / tau, top_p)
    assert 1 < mask.sum() < 9
    want = np.where(mask, q, 0.0) / q[mask].sum()
    counts = np.zeros(9)
    n = 8000
    for step in range(n):
        g = orc.gumbel_noise(orc.sampling_uniforms(21, step, 2, 1, 9))
        counts[orc.sampled_token(logits, tau, g, top_p)[0]] += 1
    assert counts[~mask].sum() == 0
    assert scipy.stats.chisquare(counts[mask], want[mask] * n)[1] > 1e-3
    assert scipy.stats.chisquare(counts[mask], q[mask] / q[mask].sum() * n * 1.0)[1] > 1e-3
    # and not the unrestricted distribution (which puts mass outside the set)
    assert q[~mask].sum() > 0.05


def test_verify_with_nucleus_sampling():
    wl = wk.Workload("nuc", d=32, V=60, dtype="f32", B=2, T=3, K=5, p=0.2, bonus=True, data_seed=17)
    W, h, seeds = wk.make_weight(wl, sigma=0.4), wk.make_hidden(wl), wk.make_seeds(wl, base_seed=2)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    tau, top_p = 1.2, 0.6
    out = orc.verify(h, W, draft, seeds, wl.K, wl.p, temperature=tau, top_p=top_p, want_logits=(0, wl.V))
    L = out["logits"].reshape(wl.B, wl.T, wl.K, wl.V)
    inside = 0
    for b in range(wl.B):
        for t in range(wl.T):
            for i in range(wl.K):
                q = scipy.special.softmax(L[b, t, i] / tau)
                order = np.argsort(-q, kind="stable")
                n = int(np.argmax(np.cumsum(q[order]) >= top_p)) + 1
                keep = q >= q[order[n - 1]]
                g = scipy.stats.gumbel_r.ppf(orc.sampling_uniforms(seeds[b], 0, t, i, wl.V))
                y = np.where(keep, L[b, t, i] / tau + g, -np.inf)
                assert out["path_ids"][b, t, i] == int(np.argmax(y))
                inside += int(keep.sum())
    assert inside < wl.B * wl.T * wl.K * wl.V            # the truncation did cut something
    free = orc.verify(h, W, draft, seeds, wl.K, wl.p, temperature=tau)
    assert (free["path_ids"] != out["path_ids"]).any()
    assert np.array_equal(orc.verify(h, W, draft, seeds, wl.K, wl.p, temperature=tau, top_p=1.0)["path_ids"], free["path_ids"])
