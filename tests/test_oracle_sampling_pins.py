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
