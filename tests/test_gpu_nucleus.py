"""Sampled path tokens restricted to the nucleus (top-p set), HIP path against the oracle through the C ABI.

The nucleus boundary is decided by a running sum of probabilities and the draw by an arg max of
perturbed logits; the GPU does both in float32 (masses as 64-bit integers), the oracle in float64.
What is unique is checked exactly, the rest for validity:
  * the GPU's token lies inside the largest nucleus the tolerances allow,
  * it beats (to within the perturbed-value tolerance) every token of the smallest one,
  * where boundary and winner are clear of the tolerances it IS the oracle's token (counted: most rows),
  * vote / hit / accepted length follow bit-exactly from the GPU's own path tokens.
Tolerances: logits carry about 1e-5 absolute error (fp32 accumulation of bf16 products), i.e.
1e-5 / tau on z = l / tau; the mass fractions inherit a relative error of that size, bounded here by
MASS_EPS; perturbed values within PERT_TOL * max(1, 1 / tau) count as tied."""
import numpy as np
import pytest

from oracle import dropmatch_oracle as orc
from paper_2603_03333_amd import workloads as wk

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2603_03333_amd import binding as dmb  # noqa: E402
from gpu_harness import Runner, check_graph_replays, to_device  # noqa: E402

MASS_EPS = 1e-4
Z_DELTA = 5e-5
PERT_TOL = 1e-3


@pytest.fixture(scope="module")
def runner():
    r = Runner(max_rows=2048, max_d=512, max_V=8192)
    r.reserve_js(max_positions=128, max_K=64)
    yield r
    r.close()


def check_nucleus_tokens(gpu_ids, logits, seeds, step, tau, top_p, B, T, K, KU, t0=0):
    """gpu_ids [B,T,K], logits [B*T*K, V] (oracle, float64); t0: position of row 0 in the call the
    tokens come from (the noise is keyed on it).  Returns (#rows, #rows equal to the oracle's draw)."""
    f = max(1.0, 1.0 / tau)
    rows = same = 0
    for b in range(B):
        for t in range(T):
            for i in range(KU):
                z = logits[(b * T + t) * K + i] / tau
                V = z.size
                y = z + orc.gumbel_noise(orc.sampling_uniforms(seeds[b], step, t0 + t, i, V))
                q = orc.softmax(z)
                order = np.argsort(-q, kind="stable")
                cum = np.cumsum(q[order])
                n_lo = min(int(np.searchsorted(cum, top_p - MASS_EPS, side="left")) + 1, V)
                n_hi = min(int(np.searchsorted(cum, top_p + MASS_EPS, side="left")) + 1, V)
                sure = z >= z[order[n_lo - 1]] + Z_DELTA * f          # inside whatever the rounding does
                maybe = z >= z[order[n_hi - 1]] - Z_DELTA * f         # the largest set the tolerances allow
                tok = int(gpu_ids[b, t, i])
                assert 0 <= tok < V and maybe[tok], f"row ({b},{t},{i}): token {tok} lies outside the nucleus"
                if sure.any():
                    assert y[tok] >= y[sure].max() - PERT_TOL * f, f"row ({b},{t},{i}): token {tok} is not the best of the nucleus"
                want, gap = orc.sampled_token(logits[(b * T + t) * K + i], tau, y - z, top_p)
                clear = (sure.sum() == maybe.sum()) and gap >= PERT_TOL * f
                if clear:
                    assert tok == want, f"row ({b},{t},{i}): {tok} != {want} at a row clear of every tolerance"
                rows += 1
                same += int(tok == want)
    return rows, same


def _run(runner, wl, W, h, seeds, draft, tau, top_p, step=0, rule=orc.RULE_ANY, flags=0, parent=None):
    ref = orc.verify(h, W, draft, seeds, wl.K, wl.p, rule=rule, step=step, parent=parent, temperature=tau, top_p=top_p,
                     clean_last_path=bool(flags & dmb.DM_FLAG_CLEAN_LAST_PATH), want_logits=(0, wl.V))
    res = runner.verify(wl, to_device(h, wl.dtype), to_device(W, wl.dtype), draft, seeds, rule=rule, step=step,
                        flags=flags | dmb.DM_FLAG_SAMPLE_PATHS, parent=parent, temperature=tau, top_p=top_p)
    KU = wl.K - 1 if flags & dmb.DM_FLAG_CLEAN_LAST_PATH else wl.K
    rows, same = check_nucleus_tokens(res["path_ids"], ref["logits"], seeds, step, tau, top_p, wl.B, wl.T, wl.K, KU)
    exp = orc.acceptance_from_path_ids(res["path_ids"][:, :, :KU], draft, rule, parent)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], exp[k]), k
    return ref, res, rows, same


@pytest.mark.parametrize("d,V,B,T,K,dtype,tau,top_p", [
    (256, 3000, 1, 8, 16, "bf16", 1.0, 0.9),     # W-streaming kernel, ragged last vocabulary chunk
    (256, 4096, 2, 6, 16, "bf16", 0.7, 0.5),     # 256 x 256 tiles
    (100, 130, 2, 3, 5, "f32", 1.5, 0.8),        # generic kernel, K not a multiple of 4
    (128, 777, 1, 3, 12, "bf16", 0.25, 0.95),    # K4 = 12: thread mapping padded to 16 paths
    (64, 2049, 3, 2, 33, "bf16", 1.0, 0.3),      # 33 paths: 64-wide mapping, one vocabulary row past a chunk
    (128, 1500, 1, 4, 64, "bf16", 2.0, 0.99),    # the most paths the variant takes
    (256, 3000, 1, 8, 16, "bf16", 50.0, 0.5),    # nearly uniform: distances of ~1e-5 in l / tau against the 2^-19 search key
    (256, 3000, 2, 4, 16, "bf16", 0.05, 0.9),    # very sharp: most tokens beyond the range of the key (no mass)
    (256, 3000, 1, 8, 16, "bf16", 2.5, 0.9),     # from temperature 2 on: fine bins next to the maximum; a flat row, threshold in them
    (256, 3000, 2, 4, 8, "bf16", 2.0, 0.15),     # the same with a small nucleus
    (128, 1500, 1, 4, 40, "bf16", 3.0, 0.7),     # 40 paths: too many for the fine bins (coarse ones only)
])
def test_nucleus_tokens_flat_distributions(runner, d, V, B, T, K, dtype, tau, top_p):
    wl = wk.Workload("nuc", d=d, V=V, dtype=dtype, B=B, T=T, K=K, p=0.2, bonus=True, data_seed=d + V + K)
    W, h = wk.make_weight(wl), wk.make_hidden(wl)
    seeds = wk.make_seeds(wl, base_seed=23)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    for rule, step in ((orc.RULE_ANY, 0), (orc.RULE_MAJORITY, 9)):
        ref, res, rows, same = _run(runner, wl, W, h, seeds, draft, tau, top_p, step=step, rule=rule)
        print(f"[nucleus {dtype} M={B*T*K} V={V} tau={tau} top_p={top_p}] rows={rows} equal to the oracle's draw={same}", flush=True)
        assert same >= 0.9 * rows


def test_nucleus_tokens_peaked_distributions(runner):
    """Planted dominant tokens (the shape of a real LM's next-token distribution): small nuclei."""
    wl = wk.Workload("nucp", d=256, V=4096, dtype="bf16", B=2, T=6, K=8, p=0.1, bonus=False, data_seed=77)
    W = wk.make_weight(wl, sigma=0.1)
    h, planted = wk.make_planted_hidden(wl, W, alpha=9.0)
    seeds = wk.make_seeds(wl, base_seed=3)
    draft = planted.copy()
    for top_p, tau in ((0.5, 1.0), (0.9, 1.0), (0.9, 2.5), (0.999, 2.0)):   # temperature >= 2: fine bins, thresholds beyond them
        ref, res, rows, same = _run(runner, wl, W, h, seeds, draft, tau, top_p)
        sizes = [int(orc.nucleus(ref["logits"][r] / tau, top_p)[0].sum()) for r in range(0, rows, 7)]
        print(f"[nucleus peaked top_p={top_p} tau={tau}] rows={rows} equal={same} nucleus sizes (sample)={sizes[:8]}", flush=True)
        assert same >= 0.9 * rows and (tau > 1.0 or max(sizes) < wl.V // 4)


@pytest.mark.parametrize("B,T,K", [(1, 8, 16), (3, 6, 16)])     # W-streaming kernel / 256 x 256 kernel in store mode
def test_nucleus_verify_can_be_captured_in_a_hip_graph(runner, B, T, K):
    """The four nucleus launches keep state between calls (bins, list counts and the second key array
    cleared by the scan): replayed from a HIP graph they must leave it as an eager call
    does.  Every replay equals the eager call, with eager calls on other inputs in between."""
    wl = wk.Workload("nucg", d=256, V=3000, dtype="bf16", B=B, T=T, K=K, p=0.1, bonus=True, data_seed=91 + B)
    W, h, seeds = wk.make_weight(wl, sigma=0.1), wk.make_hidden(wl), wk.make_seeds(wl, base_seed=5)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    kw = dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=0.9, top_p=0.8)
    eager = runner.verify(wl, hd, Wd, draft, seeds, **kw)
    prm, keep = runner.params(wl, seeds, **kw)
    draft_dev = torch.from_numpy(draft).cuda()
    out = dict(accept_len=torch.zeros(B, dtype=torch.int32, device="cuda"),
               hit=torch.zeros((B, T), dtype=torch.uint8, device="cuda"),
               path_ids=torch.zeros((B, T, K), dtype=torch.int32, device="cuda"),
               vote_ids=torch.zeros((B, T), dtype=torch.int32, device="cuda"))

    def between():
        other = runner.verify(wl, hd, Wd, draft, seeds, step=3, flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=0.9, top_p=0.5)
        assert (other["path_ids"] != eager["path_ids"]).any()

    check_graph_replays(lambda st: dmb.dropmatch_verify(runner.ctx, prm, hd, Wd, draft_dev, stream=st, **out),
                        out, eager, between)


@pytest.mark.parametrize("K,classes,top_p,tau", [
    (16, (1.0, 0.5), 0.5, 1.0),        # 1500 tied tokens per class: the stage of a draw workgroup runs over
    (4, (1.0, 0.5), 0.9, 1.0),         # 4 paths: the stages hold everything, the row's list itself runs over
    (8, (1.0, 0.96875, 0.5), 0.7, 2.0),  # two classes share the leading digit of the threshold
    (8, (0.0,), 0.6, 1.0),             # all logits equal (W = 0): the nucleus is the whole vocabulary
])
def test_nucleus_rows_whose_candidate_list_does_not_fit(runner, K, classes, top_p, tau):
    """Few distinct logit values per row: thousands of tokens share the leading digit of the threshold, more
    than a row's candidate list (max(1024, max_V / 8) entries) takes; such rows read their candidates
    from the logit store.  W[v] = c[v mod n] * w0, so the logits of a row are c[v mod n] * (w0 . h~)."""
    wl = wk.Workload("nucfit", d=128, V=3000, dtype="bf16", B=2, T=3, K=K, p=0.25, bonus=True, data_seed=404 + K)
    w0 = wk.make_weight(wl.with_(V=1), sigma=0.1)[0]
    c = np.asarray(classes, dtype=np.float32)
    W = wk.round_to_bf16(c[np.arange(wl.V) % c.size][:, None] * w0[None, :])
    h = wk.make_hidden(wl)
    seeds = wk.make_seeds(wl, base_seed=8)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    for step in (0, 5):
        ref, res, rows, same = _run(runner, wl, W, h, seeds, draft, tau, top_p, step=step)
        print(f"[nucleus tied classes K={K} classes={classes}] rows={rows} equal to the oracle's draw={same}", flush=True)
        assert same >= 0.9 * rows
    # an ordinary call right after leaves no trace of the long lists
    W2 = wk.make_weight(wl, sigma=0.1)
    _run(runner, wl, W2, h, seeds, wk.make_draft_ids(wl, orc.greedy_ids(h, W2)), tau, top_p)


def test_nucleus_candidate_list_longer_than_the_registers_hold():
    """A list that fits its row's capacity (max_V / 8 = 5000 entries) but not the 4096 entries the last pass
    holds in registers: it is walked in memory.  Every 9th token shares one logit (W[v] = w0), the others
    are small Gaussian rows, so where w0 . h~ > 0 the 4445 tied tokens are the top of the row and share
    the leading digit of the threshold; 115 of them per 1024-row chunk stay below the 128 a draw workgroup
    stages per path."""
    wl = wk.Workload("nuclong", d=128, V=40000, dtype="bf16", B=1, T=3, K=4, p=0.2, bonus=True, data_seed=911)
    r = Runner(max_rows=64, max_d=128, max_V=wl.V)
    try:
        r.reserve_js(max_positions=wl.B * wl.T, max_K=wl.K)
        w0 = wk.make_weight(wl.with_(V=1), sigma=0.1)[0]
        W = wk.make_weight(wl, sigma=0.01)
        W[::9] = w0[None, :]
        h = wk.make_hidden(wl)
        h[:, 1:] = wk.round_to_bf16(h[:, 1:] + 2.0 * w0)       # positions 1, 2: w0 . h~ > 0 on (nearly) every path
        seeds = wk.make_seeds(wl, base_seed=2)
        draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
        for top_p, tau in ((0.5, 1.0), (0.05, 0.7), (0.97, 1.3)):
            ref, res, rows, same = _run(r, wl, W, h, seeds, draft, tau, top_p)
            tied_top = sum(int(np.argmax(ref["logits"][x]) % 9 == 0) for x in range(rows))
            print(f"[nucleus long list top_p={top_p}] rows={rows} equal={same} rows whose top is the tied class={tied_top}", flush=True)
            assert same >= 0.9 * rows and tied_top >= 6
    finally:
        r.close()


def test_nucleus_limits_and_options(runner):
    wl = wk.Workload("nucl", d=128, V=1000, dtype="bf16", B=2, T=5, K=8, p=0.3, bonus=True, data_seed=5)
    W, h = wk.make_weight(wl, sigma=0.05), wk.make_hidden(wl)
    seeds = wk.make_seeds(wl, base_seed=11)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    flag = dmb.DM_FLAG_SAMPLE_PATHS
    plain = runner.verify(wl, hd, Wd, draft, seeds)
    free = runner.verify(wl, hd, Wd, draft, seeds, flags=flag, temperature=0.9)
    # top_p = 1 and 0 are the unrestricted draw (the same code path), a vanishing top_p is the arg max
    for tp in (1.0, 0.0):
        assert np.array_equal(runner.verify(wl, hd, Wd, draft, seeds, flags=flag, temperature=0.9, top_p=tp)["path_ids"],
                              free["path_ids"])
    tiny = runner.verify(wl, hd, Wd, draft, seeds, flags=flag, temperature=0.9, top_p=1e-7)
    assert np.array_equal(tiny["path_ids"], plain["path_ids"])
    # all but a sliver of the mass: nearly always the unrestricted draw, and never an invalid token
    wide = runner.verify(wl, hd, Wd, draft, seeds, flags=flag, temperature=0.9, top_p=0.99999)
    assert (wide["path_ids"] == free["path_ids"]).mean() > 0.95
    # reproducible, also right after a call with other parameters
    a = runner.verify(wl, hd, Wd, draft, seeds, flags=flag, temperature=0.9, top_p=0.6)
    runner.verify(wl, hd, Wd, draft, seeds, flags=flag, temperature=0.5, top_p=0.2, step=3)
    b = runner.verify(wl, hd, Wd, draft, seeds, flags=flag, temperature=0.9, top_p=0.6)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    # a clean last path keeps its arg max and stays out of the rules; a tree works like a chain
    _run(runner, wl, W, h, seeds, draft, 0.9, 0.6, flags=dmb.DM_FLAG_CLEAN_LAST_PATH)
    c = runner.verify(wl, hd, Wd, draft, seeds, flags=flag | dmb.DM_FLAG_CLEAN_LAST_PATH, temperature=0.9, top_p=0.6)
    assert np.array_equal(c["path_ids"][:, :, -1], orc.greedy_ids(h, W))
    wt = wl.with_(tree=True, bonus=False)
    parent = wk.make_tree_parents(wt, max_depth=3, max_branch=2)
    _run(runner, wt, W, h, seeds, wk.make_tree_draft_ids(wt, parent, orc.greedy_ids(h, W)), 0.9, 0.6, parent=parent,
         rule=orc.RULE_MAJORITY)


def test_nucleus_needs_the_reserved_store():
    r = Runner(max_rows=64, max_d=64, max_V=64)
    try:
        wl = wk.Workload("nucr", d=64, V=64, dtype="bf16", B=1, T=2, K=4, p=0.1, data_seed=1)
        W, h = wk.make_weight(wl), wk.make_hidden(wl)
        seeds, draft = wk.make_seeds(wl), np.zeros((1, 2), dtype=np.int32)
        with pytest.raises(dmb.DropMatchError, match="dm_reserve_js"):
            r.verify(wl, to_device(h, "bf16"), to_device(W, "bf16"), draft, seeds, flags=dmb.DM_FLAG_SAMPLE_PATHS,
                     temperature=1.0, top_p=0.5)
        r.reserve_js(max_positions=1, max_K=4)
        with pytest.raises(dmb.DropMatchError, match="exceed"):
            r.verify(wl, to_device(h, "bf16"), to_device(W, "bf16"), draft, seeds, flags=dmb.DM_FLAG_SAMPLE_PATHS,
                     temperature=1.0, top_p=0.5)
        r.reserve_js(max_positions=2, max_K=4)
        r.verify(wl, to_device(h, "bf16"), to_device(W, "bf16"), draft, seeds, flags=dmb.DM_FLAG_SAMPLE_PATHS,
                 temperature=1.0, top_p=0.5)
    finally:
        r.close()


@pytest.fixture(scope="module")
def small_runner():
    r = Runner(max_rows=1024, max_d=512, max_V=4096)
    r.reserve_js(max_positions=64, max_K=64)
    yield r
    r.close()


@pytest.mark.parametrize("case", range(24))
def test_random_nucleus_case(small_runner, case):
    """Seeded random shapes and options: vocabularies from 1 token up, 1 to 64 paths, both storage types,
    flat and peaked distributions, top_p from 1e-6 to 0.999, clean last path, shared masks."""
    rng = np.random.default_rng(52000 + case)
    bf16 = rng.random() < 0.75
    d = int(rng.choice([64, 128, 192, 256, 512])) if (bf16 and rng.random() < 0.8) else int(rng.integers(5, 200))
    V = int(rng.choice([1, 2, 3, 7, 255, 256, 257, 1000, 2049, 4096]) if rng.random() < 0.5 else rng.integers(2, 3000))
    K = int(rng.choice([1, 2, 3, 5, 8, 12, 16, 17, 32, 40, 64]))
    T = int(rng.integers(1, 10))
    B = int(rng.integers(1, 5))
    while B * T * K > 1024 or B * T > 64:
        T = max(1, T - 1)
        B = max(1, B - 1)
    p = float(rng.choice([0.0, 0.1, 0.3, 0.5]))
    tau = float(rng.choice([0.3, 0.8, 1.0, 2.0]))
    top_p = float(rng.choice([1e-6, 0.05, 0.3, 0.5, 0.8, 0.9, 0.95, 0.999]))
    clean = K >= 2 and rng.random() < 0.3
    peaked = rng.random() < 0.4
    dtype = "bf16" if bf16 else "f32"
    wl = wk.Workload(f"n{case}", d=d, V=V, dtype=dtype, B=B, T=T, K=K, p=p, bonus=bool(rng.integers(0, 2)),
                     data_seed=33000 + case)
    W = wk.make_weight(wl, sigma=0.1)
    h = wk.make_planted_hidden(wl, W, alpha=8.0)[0] if peaked else wk.make_hidden(wl)
    seeds = rng.integers(0, 2 ** 63, size=B, dtype=np.uint64)
    step = int(rng.integers(0, 2 ** 32))
    rule = int(rng.integers(0, 2))
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    flags = (dmb.DM_FLAG_CLEAN_LAST_PATH if clean else 0) | (dmb.DM_FLAG_FORCE_GENERIC if rng.random() < 0.2 else 0) | \
            (dmb.DM_FLAG_SHARE_MASK_ACROSS_POS if rng.random() < 0.3 else 0)
    ref = orc.verify(h, W, draft, seeds, K, p, rule=rule, step=step, temperature=tau, top_p=top_p, clean_last_path=clean,
                     share_mask_across_pos=bool(flags & dmb.DM_FLAG_SHARE_MASK_ACROSS_POS), want_logits=(0, V))
    res = small_runner.verify(wl, to_device(h, dtype), to_device(W, dtype), draft, seeds, rule=rule, step=step,
                              flags=flags | dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau, top_p=top_p)
    KU = K - 1 if clean else K
    rows, same = check_nucleus_tokens(res["path_ids"], ref["logits"], seeds, step, tau, top_p, B, T, K, KU)
    exp = orc.acceptance_from_path_ids(res["path_ids"][:, :, :KU], draft, rule, None)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], exp[k]), f"case {case}: {k}"
    if clean:
        assert np.array_equal(res["path_ids"][:, :, -1], orc.greedy_ids(h, W))
    assert same >= 0.9 * rows, f"case {case}: only {same} of {rows} rows equal the oracle's draw"
