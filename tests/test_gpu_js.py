"""Parity of the distribution-level rules (Eq. 5, Eq. 6, Algorithm 1) on the HIP path with the CPU
oracle, through the C ABI.  Bars: path tokens / votes as in the token-level tests; JS values within
JS_ATOL + JS_RTOL * |JS| (derivation in gpu_harness); per-row decisions and accept lengths equal
to the oracle's, except that at rows whose Eq. (6) margin lies inside the tolerance band the
GPU's own float32 comparison is taken (counted, printed) and the acceptance is re-derived from
it with the oracle's rule logic."""
import numpy as np
import pytest

from oracle import dropmatch_oracle as orc
from paper_2603_03333_amd import workloads as wk

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2603_03333_amd import binding as dmb  # noqa: E402
from gpu_harness import Runner, check_graph_replays, compare_js, compare_path_ids, to_device  # noqa: E402


@pytest.fixture(scope="module")
def runner():
    r = Runner(max_rows=4096, max_d=4096, max_V=8192)
    r.reserve_js(max_positions=64, max_K=64)
    yield r
    r.close()


def _problem(d, V, dtype, B, T, K, p, seed, bonus=True, planted=0.0, topk=0, sigma=0.02):
    wl = wk.Workload("js", d=d, V=V, dtype=dtype, B=B, T=T, K=K, p=p, bonus=bonus, data_seed=seed)
    W = wk.make_weight(wl, sigma=sigma)
    h = wk.make_planted_hidden(wl, W, planted)[0] if planted else wk.make_hidden(wl)
    seeds = wk.make_seeds(wl, base_seed=29)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    clean = np.einsum("vd,btd->btv", W.astype(np.float64), h.astype(np.float64)).astype(np.float32)
    probs = wk.make_draft_probs(wl, clean, topk=topk)
    return wl, W, h, seeds, draft, probs


def _check(runner, wl, W, h, seeds, draft, probs, rule, label):
    o_rule = orc.RULE_JS if rule == dmb.DM_RULE_JS else orc.RULE_JS_OR_MAJORITY
    ref = orc.verify_js(h, W, draft, probs, seeds, wl.K, wl.p, rule=o_rule)
    hd, Wd = to_device(h, wl.dtype), to_device(W, wl.dtype)
    res = runner.verify_js(wl, hd, Wd, draft, probs, seeds, rule=rule)
    nflip, nnear = compare_path_ids(res["path_ids"], ref)
    votes = orc.acceptance_from_path_ids(res["path_ids"], draft, orc.RULE_MAJORITY)
    assert np.array_equal(res["vote_ids"], votes["vote_ids"]) and np.array_equal(res["vote_cnt"], votes["vote_cnt"])
    n_tie, gpu_js = compare_js(res, ref, draft, rule == dmb.DM_RULE_JS, nflip, label)
    want_hit = gpu_js.copy()
    if rule == dmb.DM_RULE_JS_OR_MAJORITY:
        want_hit |= votes["hit"].astype(bool)
    assert np.array_equal(res["hit"].astype(bool), want_hit), f"{label}: hit"
    exp = orc.acceptance_from_hits(want_hit)
    for k in ("accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], exp[k]), f"{label}: {k}"
    if n_tie == 0 and nflip == 0:       # then everything must equal the oracle's own outputs
        for k in ("hit", "accept_mask", "accept_len", "best_node"):
            assert np.array_equal(res[k], ref[k]), f"{label}: {k} vs oracle"
    return ref, res


@pytest.mark.parametrize("rule", [dmb.DM_RULE_JS, dmb.DM_RULE_JS_OR_MAJORITY])
def test_tiny_config_fp32_generic_kernel(runner, rule):
    wl = wk.CONFIGS["tiny"]
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    clean = np.einsum("vd,btd->btv", W.astype(np.float64), h.astype(np.float64)).astype(np.float32)
    probs = wk.make_draft_probs(wl, clean)
    _check(runner, wl, W, h, seeds, draft, probs, rule, f"tiny/f32 rule={rule}")


@pytest.mark.parametrize("d,V,B,T,K,p", [
    (256, 4096, 1, 6, 5, 0.3),      # the paper's operating point K = 5, p = 0.3 (K4 = 8)
    (512, 5000, 2, 4, 16, 0.1),     # three vocabulary chunks, the last one ragged
    (256, 1000, 1, 3, 1, 0.2),      # K = 1: the centroid is the single head, radius 0
    (128, 2048, 1, 2, 33, 0.1),     # K4 = 36 -> widest register tile of the JS kernels
    (256, 3000, 4, 8, 12, 0.2),     # 384 rows: the 256 x 256 MFMA kernel stores the logits
    (192, 777, 1, 5, 64, 0.05),     # K = 64, the limit
])
def test_bf16_mfma_shapes(runner, d, V, B, T, K, p):
    wl, W, h, seeds, draft, probs = _problem(d, V, "bf16", B, T, K, p, seed=300 + K)
    _check(runner, wl, W, h, seeds, draft, probs, dmb.DM_RULE_JS_OR_MAJORITY, f"bf16 d={d} V={V} B={B} T={T} K={K}")


def test_peaked_heads_majority_branch(runner):
    """Planted dominant tokens: heads agree, the cluster is tight, Eq. (6) rejects drafts that are
    close but not inside, and Algorithm 1's second branch (Eq. 7) accepts matching tokens."""
    wl, W, h, seeds, draft, probs = _problem(256, 4096, "bf16", 2, 6, 5, 0.3, seed=410, planted=12.0, sigma=0.05)
    ref, res = _check(runner, wl, W, h, seeds, draft, probs, dmb.DM_RULE_JS_OR_MAJORITY, "planted")
    js_only = orc.verify_js(h, W, draft, probs, seeds, wl.K, wl.p, rule=orc.RULE_JS)
    assert ref["hit"].sum() > js_only["hit"].sum(), "the probe should exercise the majority branch"


def test_truncated_draft_distribution_has_zeros(runner):
    wl, W, h, seeds, draft, probs = _problem(256, 4096, "bf16", 1, 4, 8, 0.1, seed=420, topk=50)
    assert (probs == 0).any()
    _check(runner, wl, W, h, seeds, draft, probs, dmb.DM_RULE_JS, "topk-50 draft")


def test_p_zero_cluster_collapses(runner):
    wl, W, h, seeds, draft, probs = _problem(256, 2048, "bf16", 1, 4, 8, 0.0, seed=430)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    res = runner.verify_js(wl, hd, Wd, draft, probs, seeds, rule=dmb.DM_RULE_JS_OR_MAJORITY)
    assert np.all(np.abs(res["js_heads"]) < 1e-6)
    greedy = orc.greedy_ids(h, W)
    assert np.array_equal(res["hit"].astype(bool), (draft == greedy) & (draft >= 0))


def test_js_is_deterministic_and_optional_outputs(runner):
    wl, W, h, seeds, draft, probs = _problem(256, 4096, "bf16", 2, 4, 8, 0.1, seed=440)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    a = runner.verify_js(wl, hd, Wd, draft, probs, seeds)
    b = runner.verify_js(wl, hd, Wd, draft, probs, seeds)
    for k in a:
        assert np.array_equal(a[k], b[k], equal_nan=True), k
    prm, keep = runner.params(wl, seeds, rule=dmb.DM_RULE_JS)
    acc = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
    dmb.dropmatch_verify_js(runner.ctx, prm, hd, Wd, torch.from_numpy(draft).cuda(),
                            torch.from_numpy(probs).cuda(), acc)
    torch.cuda.synchronize()
    only = runner.verify_js(wl, hd, Wd, draft, probs, seeds, rule=dmb.DM_RULE_JS)
    assert np.array_equal(acc.cpu().numpy(), only["accept_len"])


@pytest.mark.parametrize("B,T,K", [(1, 6, 8), (4, 6, 16)])     # W-streaming kernel / 256 x 256 kernel in store mode
def test_verify_js_can_be_captured_in_a_hip_graph(runner, B, T, K):
    """Store-mode contraction, both JS passes and the acceptance step replayed from a HIP graph: every
    replay equals the eager call, with other eager calls (which overwrite the stored logits and the
    partial sums) in between."""
    wl, W, h, seeds, draft, probs = _problem(256, 3000, "bf16", B, T, K, 0.1, seed=450 + K)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    eager = runner.verify_js(wl, hd, Wd, draft, probs, seeds)
    prm, keep = runner.params(wl, seeds, rule=dmb.DM_RULE_JS_OR_MAJORITY)
    draft_dev, probs_dev = torch.from_numpy(draft).cuda(), torch.from_numpy(probs).cuda()
    out = dict(accept_len=torch.zeros(B, dtype=torch.int32, device="cuda"),
               hit=torch.zeros((B, T), dtype=torch.uint8, device="cuda"),
               path_ids=torch.zeros((B, T, K), dtype=torch.int32, device="cuda"),
               js_draft=torch.zeros((B, T), dtype=torch.float32, device="cuda"),
               js_heads=torch.zeros((B, T, K), dtype=torch.float32, device="cuda"))

    def between():
        other = runner.verify_js(wl, hd, Wd, draft, probs, seeds, step=5)
        assert (other["path_ids"] != eager["path_ids"]).any()

    check_graph_replays(lambda st: dmb.dropmatch_verify_js(runner.ctx, prm, hd, Wd, draft_dev, probs_dev, stream=st, **out),
                        out, eager, between)


def test_js_argument_errors(runner):
    wl, W, h, seeds, draft, probs = _problem(64, 256, "bf16", 1, 2, 4, 0.1, seed=450)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    dd, pd = torch.from_numpy(draft).cuda(), torch.from_numpy(probs).cuda()
    acc = torch.zeros(1, dtype=torch.int32, device="cuda")
    prm, keep = runner.params(wl, seeds, rule=dmb.DM_RULE_ANY)
    with pytest.raises(dmb.DropMatchError):           # token-level rule through the JS entry point
        dmb.dropmatch_verify_js(runner.ctx, prm, hd, Wd, dd, pd, acc)
    prm, keep = runner.params(wl, seeds, rule=dmb.DM_RULE_JS)
    with pytest.raises(dmb.DropMatchError):           # JS rule through the token-level entry point
        dmb.dropmatch_verify(runner.ctx, prm, hd, Wd, dd, acc)
    with pytest.raises(dmb.DropMatchError):           # no draft distribution
        dmb.dropmatch_verify_js(runner.ctx, prm, hd, Wd, dd, None, acc)
    par = torch.tensor([[-1, 0]], dtype=torch.int32, device="cuda")
    prm, keep = runner.params(wl, seeds, rule=dmb.DM_RULE_JS, parent=par)
    with pytest.raises(dmb.DropMatchError):           # trees are not defined for these rules
        dmb.dropmatch_verify_js(runner.ctx, prm, hd, Wd, dd, pd, acc)
    fresh = Runner(max_rows=64, max_d=64, max_V=256)
    try:
        prm, keep = fresh.params(wl, seeds, rule=dmb.DM_RULE_JS)
        with pytest.raises(dmb.DropMatchError):       # dm_reserve_js was never called
            dmb.dropmatch_verify_js(fresh.ctx, prm, hd, Wd, dd, pd, acc)
        fresh.reserve_js(1, 4)
        with pytest.raises(dmb.DropMatchError):       # two positions > the one reserved
            dmb.dropmatch_verify_js(fresh.ctx, prm, hd, Wd, dd, pd, acc)
    finally:
        fresh.close()


def test_js_size_limits():
    # DM_MAX_K_JS paths and DM_MAX_TK_JS path tokens per sequence
    wl, W, h, seeds, draft, probs = _problem(64, 300, "bf16", 1, 128, 64, 0.2, seed=460, sigma=0.3)
    r = Runner(max_rows=wl.rows, max_d=wl.d, max_V=wl.V)
    try:
        r.reserve_js(wl.B * wl.T, wl.K)
        _check(r, wl, W, h, seeds, draft, probs, dmb.DM_RULE_JS_OR_MAJORITY, "js limits T*K=8192 K=64")
        for kw in (dict(K=65, T=4), dict(T=129)):
            prm, keep = r.params(wl.with_(**kw), seeds, rule=dmb.DM_RULE_JS)
            st, msg = dmb.dm_validate(prm)
            assert st == dmb.DM_EINVAL and msg
    finally:
        r.close()


@pytest.mark.parametrize("K", [5, 16, 17])
def test_js_with_clean_last_path(runner, K):
    """K-1 dropout heads form the cluster, path K-1 is the plain head (K = 17: 16 heads, the fully
    populated lane layout of the JS kernels, next to a clean 17th row)."""
    wl, W, h, seeds, draft, probs = _problem(256, 3000, "bf16", 2, 4, K, 0.2, seed=470 + K)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    flag = dmb.DM_FLAG_CLEAN_LAST_PATH
    ref = orc.verify_js(h, W, draft, probs, seeds, K, wl.p, rule=orc.RULE_JS_OR_MAJORITY, clean_last_path=True)
    res = runner.verify_js(wl, hd, Wd, draft, probs, seeds, rule=dmb.DM_RULE_JS_OR_MAJORITY, flags=flag)
    nflip, _ = compare_path_ids(res["path_ids"], ref)
    assert np.array_equal(res["path_ids"][:, :, -1], orc.greedy_ids(h, W))
    assert np.all(res["js_heads"][:, :, -1] == 0)
    n_tie, gpu_js = compare_js(res, ref, draft, False, nflip, f"js clean K={K}")
    fewer = runner.verify_js(wl.with_(K=K - 1), hd, Wd, draft, probs, seeds, rule=dmb.DM_RULE_JS_OR_MAJORITY, K=K - 1)
    # the (K-1)-path run groups lanes differently, so its sums round differently: equal within the JS bar
    from gpu_harness import JS_ATOL, JS_RTOL
    assert np.allclose(res["js_heads"][:, :, :-1], fewer["js_heads"], atol=JS_ATOL, rtol=JS_RTOL)
    assert np.allclose(res["js_draft"], fewer["js_draft"], atol=JS_ATOL, rtol=JS_RTOL)
    for k in ("vote_ids", "vote_cnt") + (("hit", "accept_len") if n_tie == 0 else ()):
        assert np.array_equal(res[k], fewer[k]), k
    if n_tie == 0 and nflip == 0:
        for k in ("hit", "accept_mask", "accept_len", "vote_ids", "vote_cnt"):
            assert np.array_equal(res[k], ref[k]), k
