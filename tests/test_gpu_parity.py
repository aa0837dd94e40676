"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Bars: masks, hit, accept_mask, accept_len, best_node, vote bit-exact; path tokens exact
except at rows whose oracle top-2 logit gap is < 1e-3 (counted, printed); logits within
2e-2 absolute for bf16 inputs with fp32 accumulation (1e-3 for fp32 inputs)."""
import numpy as np
import pytest

from oracle import dropmatch_oracle as orc
from paper_2603_03333_amd import workloads as wk

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2603_03333_amd import binding as dmb  # noqa: E402
from gpu_harness import Runner, check_graph_replays, compare_path_ids, to_device  # noqa: E402


@pytest.fixture(scope="module")
def runner():
    r = Runner(max_rows=4096, max_d=4096, max_V=8192)
    yield r
    r.close()


def _problem(name, d, V, dtype, B, T, K, p, seed, bonus=False):
    wl = wk.Workload(name, d=d, V=V, dtype=dtype, B=B, T=T, K=K, p=p, bonus=bonus, data_seed=seed)
    W, h = wk.make_weight(wl), wk.make_hidden(wl)
    seeds = wk.make_seeds(wl, base_seed=17)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    return wl, W, h, seeds, draft


def _check_against_oracle(res, ref, draft, rule, parent=None, label=""):
    ndiff, nnear = compare_path_ids(res["path_ids"], ref, label=label)
    expect = ref if ndiff == 0 else orc.acceptance_from_path_ids(res["path_ids"], draft, rule, parent)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], expect[k]), f"{label}: {k} differs"
    return ndiff


# ------------------------------------------------------------------ masks (Eq. 1)
@pytest.mark.parametrize("d,T,K,B,p,step,share", [
    (256, 5, 8, 1, 0.1, 0, False),
    (4096, 8, 16, 1, 0.1, 0, False),
    (37, 3, 5, 2, 0.3, 7, False),       # d not a multiple of 4, 8 or 32
    (96, 4, 3, 2, 0.5, 2 ** 32 - 1, True),
    (64, 1, 1, 1, 0.0, 0, False),
])
def test_masks_bit_exact(runner, d, T, K, B, p, step, share):
    wl = wk.Workload("m", d=d, V=16, dtype="bf16", B=B, T=T, K=K, p=p)
    seeds = np.array([3 + (2 ** 40) * b + b for b in range(B)], dtype=np.uint64)
    flags = dmb.DM_FLAG_SHARE_MASK_ACROSS_POS if share else 0
    got = runner.masks(wl, seeds, step=step, flags=flags)
    want = np.stack([orc.pack_mask_bits(orc.keep_masks(int(s), step, T, K, d, p, share)) for s in seeds])
    assert got.shape == want.shape and np.array_equal(got, want)


def test_masks_many_sequences_cross_seed_chunks(runner):
    # more sequences than seeds fit in one launch (seeds travel as kernel arguments)
    wl = wk.Workload("m", d=64, V=16, dtype="f32", B=300, T=2, K=3, p=0.2)
    seeds = (np.arange(300, dtype=np.uint64) * np.uint64(2654435761)) + np.uint64(1 << 33)
    got = runner.masks(wl, seeds)
    want = np.stack([orc.pack_mask_bits(orc.keep_masks(int(s), 0, 2, 3, 64, 0.2)) for s in seeds])
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ whole step, small shapes
def test_tiny_config_fp32(runner):
    wl = wk.CONFIGS["tiny"]
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    ref = orc.verify(h, W, draft, seeds, wl.K, wl.p, want_logits=(0, wl.V))
    hd, Wd = to_device(h, "f32"), to_device(W, "f32")
    res = runner.verify(wl, hd, Wd, draft, seeds)
    _check_against_oracle(res, ref, draft, orc.RULE_ANY, label="tiny/f32")
    lg = runner.logits(wl, hd, Wd, seeds, 0, wl.V)
    assert np.abs(lg - ref["logits"]).max() < 1e-3


@pytest.mark.parametrize("d,V,B,T,K,p", [
    (256, 1000, 1, 5, 5, 0.3),     # paper's K=5, p=0.3; M=25 (one partial row tile), ragged last vocabulary tile
    (128, 777, 1, 3, 16, 0.1),     # M=48 -> two row tiles
    (512, 2049, 2, 6, 8, 0.2),     # M=96 -> three row tiles; V = 8 tiles + 1 row
    (256, 4096, 1, 8, 16, 0.1),    # M=128 exactly
    (192, 1500, 3, 6, 8, 0.05),    # M=144 -> two row blocks of 128
    (64, 300, 5, 7, 9, 0.5),       # M=315, one k slab only; two 256-row tiles
    (256, 3000, 4, 8, 20, 0.1),    # M=640 -> three 256-row tiles x 12 vocabulary tiles, several rounds
    (128, 5000, 9, 8, 32, 0.2),    # M=2304 -> nine 256-row tiles
])
@pytest.mark.parametrize("rule", [orc.RULE_ANY, orc.RULE_MAJORITY])
def test_bf16_mfma_matches_oracle(runner, d, V, B, T, K, p, rule):
    wl, W, h, seeds, draft = _problem("s", d, V, "bf16", B, T, K, p, seed=d + V, bonus=True)
    prm, _ = runner.params(wl, seeds)
    assert dmb.dm_kernel_choice(prm) == 1
    ref = orc.verify(h, W, draft, seeds, K, p, rule=rule)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    res = runner.verify(wl, hd, Wd, draft, seeds, rule=rule)
    _check_against_oracle(res, ref, draft, rule, label=f"mfma d={d} V={V} M={B*T*K}")
    # the generic kernel on the same bf16 inputs
    gen = runner.verify(wl, hd, Wd, draft, seeds, rule=rule, flags=dmb.DM_FLAG_FORCE_GENERIC)
    _check_against_oracle(gen, ref, draft, rule, label=f"generic d={d} V={V}")


@pytest.mark.parametrize("d,V", [(100, 130), (37, 65), (8, 3)])
def test_generic_odd_shapes(runner, d, V):
    for dtype in ("f32", "bf16"):
        wl, W, h, seeds, draft = _problem("o", d, V, dtype, 2, 4, 6, 0.25, seed=d * V)
        prm, _ = runner.params(wl, seeds)
        assert dmb.dm_kernel_choice(prm) == 0
        ref = orc.verify(h, W, draft, seeds, wl.K, wl.p)
        res = runner.verify(wl, to_device(h, dtype), to_device(W, dtype), draft, seeds)
        _check_against_oracle(res, ref, draft, orc.RULE_ANY, label=f"generic {dtype} d={d} V={V}")


@pytest.mark.parametrize("B,T,K", [(2, 4, 8), (5, 8, 8)])      # 64 rows (small-row kernel), 320 rows (256-row tiles)
def test_logits_values_mfma_and_generic(runner, B, T, K):
    wl, W, h, seeds, draft = _problem("l", 512, 1200, "bf16", B, T, K, 0.1, seed=5)
    v0, v1 = 250, 1200      # crosses tile borders, ends at the ragged tail
    ref = orc.verify(h, W, draft, seeds, wl.K, wl.p, want_logits=(v0, v1))["logits"]
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    for flags in (0, dmb.DM_FLAG_FORCE_GENERIC):
        got = runner.logits(wl, hd, Wd, seeds, v0, v1, flags=flags)
        assert got.shape == ref.shape and np.isfinite(got).all()
        err = np.abs(got - ref).max()
        print(f"logits max abs err (flags={flags}): {err:.3e}", flush=True)
        assert err < 2e-2


def test_logits_exact_on_integer_inputs(runner):
    # small integers: every product and partial sum is exact in bf16/fp32, so with p = 0.5
    # (scale exactly 2) the accumulator must equal the fp64 oracle bit for bit
    rng = np.random.default_rng(3)
    wl = wk.Workload("int", d=128, V=520, dtype="bf16", B=1, T=4, K=8, p=0.5)
    h = rng.integers(-4, 5, size=(1, 4, 128)).astype(np.float32)
    W = rng.integers(-3, 4, size=(520, 128)).astype(np.float32)
    seeds = np.array([11], dtype=np.uint64)
    ref = orc.verify(h, W, np.zeros((1, 4), int), seeds, wl.K, wl.p, want_logits=(0, 520))
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    for flags in (0, dmb.DM_FLAG_FORCE_GENERIC):
        got = runner.logits(wl, hd, Wd, seeds, 0, 520, flags=flags)
        assert np.array_equal(got.astype(np.float64), ref["logits"])
    res = runner.verify(wl, hd, Wd, np.zeros((1, 4), np.int32), seeds)
    assert np.array_equal(res["path_ids"], ref["path_ids"])      # exact ties resolve to the smallest index


# ------------------------------------------------------------------ fixed points on the GPU path
def test_p_zero_is_greedy_verification(runner):
    wl, W, h, seeds, _ = _problem("g", 256, 3000, "bf16", 2, 6, 8, 0.0, seed=9)
    greedy = orc.greedy_ids(h, W)
    draft = greedy.copy()
    draft[0, 4] = (draft[0, 4] + 1) % wl.V
    res = runner.verify(wl, to_device(h, "bf16"), to_device(W, "bf16"), draft, seeds)
    assert (res["path_ids"] == greedy[:, :, None]).all()
    assert (res["vote_cnt"] == wl.K).all() and res["accept_len"].tolist() == [4, 6]


def test_share_mask_flag_and_step(runner):
    wl, W, h, seeds, draft = _problem("f", 256, 1500, "bf16", 2, 5, 6, 0.3, seed=21)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    for step, share in ((0, True), (5, False), (5, True)):
        ref = orc.verify(h, W, draft, seeds, wl.K, wl.p, step=step, share_mask_across_pos=share)
        res = runner.verify(wl, hd, Wd, draft, seeds, step=step,
                            flags=dmb.DM_FLAG_SHARE_MASK_ACROSS_POS if share else 0)
        _check_against_oracle(res, ref, draft, orc.RULE_ANY, label=f"step={step} share={share}")


def test_tree_mode_matches_oracle(runner):
    wl = wk.Workload("t", d=256, V=2000, dtype="bf16", B=3, T=24, K=5, p=0.1, tree=True, data_seed=31)
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl, 2)
    parent = wk.make_tree_parents(wl, max_depth=5, max_branch=3)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    # plant tokens that some path of the parent row produces, so that deep nodes get accepted
    paths = orc.verify(h, W, np.zeros((wl.B, wl.T), int), seeds, wl.K, wl.p)["path_ids"]
    rng = np.random.default_rng(4)
    draft = wk.make_tree_draft_ids(wl, parent, orc.greedy_ids(h, W))
    for b in range(wl.B):
        for n in range(1, wl.T):
            if rng.random() < 0.6:
                draft[b, n] = paths[b, parent[b, n], rng.integers(0, wl.K)]
    for rule in (orc.RULE_ANY, orc.RULE_MAJORITY):
        ref = orc.verify(h, W, draft, seeds, wl.K, wl.p, rule=rule, parent=parent)
        res = runner.verify(wl, hd, Wd, draft, seeds, rule=rule, parent=parent)
        _check_against_oracle(res, ref, draft, rule, parent=parent, label=f"tree rule={rule}")
        assert ref["accept_len"].max() >= 2
    # a broken parent index rejects the node instead of reading out of bounds
    bad = parent.copy()
    bad[0, 5] = 7
    res = runner.verify(wl, hd, Wd, draft, seeds, parent=bad)
    assert res["hit"][0, 5] == 0 and res["accept_mask"][0, 5] == 0


def test_chain_equals_degenerate_tree_on_gpu(runner):
    wl, W, h, seeds, draft = _problem("c", 256, 1200, "bf16", 2, 7, 6, 0.05, seed=41, bonus=True)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    chain = runner.verify(wl, hd, Wd, draft, seeds)
    parent, tdraft = wk.chain_as_tree(draft)
    tree = runner.verify(wl, hd, Wd, tdraft, seeds, parent=parent)
    assert np.array_equal(chain["path_ids"], tree["path_ids"])
    assert np.array_equal(chain["accept_len"], tree["accept_len"])


def test_determinism_and_optional_outputs(runner):
    wl, W, h, seeds, draft = _problem("r", 512, 5000, "bf16", 1, 8, 16, 0.1, seed=51, bonus=True)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    first = runner.verify(wl, hd, Wd, draft, seeds)
    for _ in range(5):
        again = runner.verify(wl, hd, Wd, draft, seeds)
        for k in first:
            assert np.array_equal(first[k], again[k])
    # only the required output
    prm, keep = runner.params(wl, seeds)
    al = torch.full((wl.B,), -7, dtype=torch.int32, device="cuda")
    dmb.dropmatch_verify(runner.ctx, prm, hd, Wd, torch.from_numpy(draft).cuda(), al)
    torch.cuda.synchronize()
    assert np.array_equal(al.cpu().numpy(), first["accept_len"])


def test_works_on_a_side_stream(runner):
    wl, W, h, seeds, draft = _problem("st", 256, 1000, "bf16", 1, 4, 8, 0.1, seed=61)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    want = runner.verify(wl, hd, Wd, draft, seeds)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        got = runner.verify(wl, hd, Wd, draft, seeds)
    for k in want:
        assert np.array_equal(want[k], got[k])


def test_argument_errors_enqueue_nothing(runner):
    wl, W, h, seeds, draft = _problem("e", 64, 100, "bf16", 1, 2, 2, 0.1, seed=71)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    al = torch.zeros(1, dtype=torch.int32, device="cuda")
    dr = torch.from_numpy(draft).cuda()
    cases = [dict(p=1.0), dict(p=-0.1), dict(K=0), dict(rule=5), dict(flags=64)]
    for kw in cases:
        prm, keep = runner.params(wl, seeds, **{k: v for k, v in kw.items() if k != "K"}, K=kw.get("K"))
        if "K" in kw:
            prm.K = kw["K"]
        with pytest.raises(dmb.DropMatchError) as ei:
            dmb.dropmatch_verify(runner.ctx, prm, hd, Wd, dr, al)
        assert ei.value.status == dmb.DM_EINVAL and ei.value.message
    big = wk.Workload("big", d=64, V=100, dtype="bf16", B=1, T=64, K=128, p=0.1)   # 8192 rows > max_rows
    prm, keep = runner.params(big, [0])
    with pytest.raises(dmb.DropMatchError):
        dmb.dropmatch_verify(runner.ctx, prm, hd, Wd, dr, al)
    prm, keep = runner.params(wl, seeds)
    with pytest.raises(dmb.DropMatchError):
        dmb.dropmatch_verify(runner.ctx, prm, None, Wd, dr, al)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ edges of the shape space
@pytest.mark.parametrize("d,V,B,T,K", [
    (64, 1, 1, 1, 1),        # a single vocabulary row, a single path
    (64, 31, 1, 2, 3),       # less than one MFMA tile of vocabulary rows
    (128, 257, 1, 1, 128),   # exactly 128 rows, K larger than a wavefront
    (128, 600, 1, 1, 129),   # 129 rows: first size served by the 256-row tiles
    (64, 520, 1, 2, 128),    # exactly 256 rows
    (64, 520, 1, 1, 257),    # 257 rows -> two row tiles, second almost empty
    (64, 900, 2, 300, 1),    # many rows per sequence, one path each
])
def test_shape_edges(runner, d, V, B, T, K):
    wl, W, h, seeds, draft = _problem("edge", d, V, "bf16", B, T, K, 0.2, seed=7 * d + V + K)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    for rule in (orc.RULE_ANY, orc.RULE_MAJORITY):
        ref = orc.verify(h, W, draft, seeds, K, wl.p, rule=rule)
        res = runner.verify(wl, hd, Wd, draft, seeds, rule=rule)
        _check_against_oracle(res, ref, draft, rule, label=f"edge d={d} V={V} B={B} T={T} K={K} rule={rule}")


def test_many_paths_vote(runner):
    # K = 200 paths per row on a tiny vocabulary: many repeated tokens, modes with ties
    wl, W, h, seeds, draft = _problem("vote", 64, 7, "bf16", 2, 3, 200, 0.5, seed=99)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    for rule in (orc.RULE_ANY, orc.RULE_MAJORITY):
        ref = orc.verify(h, W, draft, seeds, 200, wl.p, rule=rule)
        res = runner.verify(wl, hd, Wd, draft, seeds, rule=rule)
        _check_against_oracle(res, ref, draft, rule, label=f"K=200 rule={rule}")
    assert res["vote_cnt"].max() > 50


def test_deep_chain_tree(runner):
    # a tree that is one long path (every node's parent is its predecessor), T = 200 nodes
    wl = wk.Workload("deep", d=64, V=50, dtype="bf16", B=2, T=200, K=4, p=0.1, tree=True, data_seed=5)
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl)
    parent = np.tile(np.arange(-1, wl.T - 1, dtype=np.int32), (wl.B, 1))
    paths = orc.verify(h, W, np.zeros((wl.B, wl.T), int), seeds, wl.K, wl.p)["path_ids"]
    draft = np.full((wl.B, wl.T), -1, dtype=np.int32)
    for b in range(wl.B):
        for n in range(1, wl.T):
            draft[b, n] = paths[b, n - 1, n % wl.K]
    draft[0, 150] = 50          # sequence 0 breaks at depth 150
    ref = orc.verify(h, W, draft, seeds, wl.K, wl.p, parent=parent)
    res = runner.verify(wl, to_device(h, "bf16"), to_device(W, "bf16"), draft, seeds, parent=parent)
    _check_against_oracle(res, ref, draft, orc.RULE_ANY, parent=parent, label="deep tree")
    assert res["accept_len"].tolist() == [149, 199]


# ------------------------------------------------------------------ the limits the header states
@pytest.mark.parametrize("d,V,B,T,K", [
    (64, 40, 1, 4096, 4),     # DM_MAX_ROWS_PER_SEQ rows and DM_MAX_TK path tokens in one sequence
    (64, 60, 1, 16, 1024),    # DM_MAX_K paths per row
])
def test_size_limits(d, V, B, T, K):
    wl, W, h, seeds, draft = _problem("limit", d, V, "bf16", B, T, K, 0.25, seed=T + K)
    r = Runner(max_rows=B * T * K, max_d=d, max_V=V)
    try:
        hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
        ref = orc.verify(h, W, draft, seeds, K, wl.p, rule=orc.RULE_MAJORITY)
        res = r.verify(wl, hd, Wd, draft, seeds, rule=orc.RULE_MAJORITY)
        _check_against_oracle(res, ref, draft, orc.RULE_MAJORITY, label=f"limit T={T} K={K}")
        # one past each limit is refused before anything is enqueued
        for kw in (dict(T=T + 1) if T == 4096 else dict(K=K + 1),):
            big = wl.with_(**kw)
            prm, keep = r.params(big, seeds)
            st, msg = dmb.dm_validate(prm)
            assert st == dmb.DM_EINVAL and msg
    finally:
        r.close()


# ------------------------------------------------------------------ HIP graph capture
@pytest.mark.parametrize("d,V,B,T,K,tau", [
    (256, 3000, 2, 6, 8, 0.0),      # W-streaming kernel, acceptance step fused into it
    (1024, 2000, 2, 6, 16, 0.7),    # 256 x 256 kernel, sampled tokens: noise scratch written and read per tile
    (256, 3000, 1, 8, 16, 1.3),     # W-streaming kernel, sampling epilogue
])
def test_verify_can_be_captured_in_a_hip_graph(runner, d, V, B, T, K, tau):
    """The step only launches kernels on the caller's stream (no allocation, no synchronisation,
    no memset), so a caller may capture it and replay it.  Every replay is checked against the
    eager result, with eager work and synchronisations between the replays."""
    wl, W, h, seeds, draft = _problem("graph", d, V, "bf16", B, T, K, 0.1, seed=321, bonus=True)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    kw = dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau) if tau else {}
    eager = runner.verify(wl, hd, Wd, draft, seeds, **kw)
    prm, keep = runner.params(wl, seeds, **kw)
    draft_dev = torch.from_numpy(draft).cuda()
    out = dict(accept_len=torch.zeros(wl.B, dtype=torch.int32, device="cuda"),
               hit=torch.zeros((wl.B, wl.T), dtype=torch.uint8, device="cuda"),
               path_ids=torch.zeros((wl.B, wl.T, wl.K), dtype=torch.int32, device="cuda"),
               vote_ids=torch.zeros((wl.B, wl.T), dtype=torch.int32, device="cuda"))

    def between():                                          # eager work between replays, other inputs
        other = runner.verify(wl, hd, Wd, draft, seeds, step=9, **kw)
        assert (other["path_ids"] != eager["path_ids"]).any()

    check_graph_replays(lambda st: dmb.dropmatch_verify(runner.ctx, prm, hd, Wd, draft_dev, stream=st, **out),
                        out, eager, between)


@pytest.mark.parametrize("d,V,B,T,K,tau", [
    (256, 3000, 2, 6, 8, 0.0),      # W-streaming kernel
    (1024, 2000, 2, 6, 16, 0.7),    # 256 x 256 kernel, sampled tokens (noise drawn by the copy wavefronts)
    (100, 130, 2, 3, 5, 1.5),       # generic kernel, sampled tokens (bf16 storage)
])
def test_graph_replays_draw_fresh_masks_from_the_device_step_word(runner, d, V, B, T, K, tau):
    """step and the seeds travel as kernel arguments, so a captured call would replay the masks it was
    captured with; with dm_params.step_dev the kernels add a word they read from device memory when they
    run.  One captured graph, the word changed between replays: every replay equals the eager call (and
    the oracle's masks) with step = base + word."""
    wl, W, h, seeds, draft = _problem("graphstep", d, V, "bf16", B, T, K, 0.2, seed=99, bonus=True)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    kw = dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau) if tau else {}
    base = 2 ** 32 - 2                                       # the sum wraps around
    word = torch.zeros(1, dtype=torch.int32, device="cuda")
    prm, keep = runner.params(wl, seeds, step=base, **kw)
    prm.step_dev = word.data_ptr()
    draft_dev = torch.from_numpy(draft).cuda()
    out = dict(accept_len=torch.zeros(wl.B, dtype=torch.int32, device="cuda"),
               hit=torch.zeros((wl.B, wl.T), dtype=torch.uint8, device="cuda"),
               path_ids=torch.zeros((wl.B, wl.T, wl.K), dtype=torch.int32, device="cuda"),
               vote_ids=torch.zeros((wl.B, wl.T), dtype=torch.int32, device="cuda"))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dmb.dropmatch_verify(runner.ctx, prm, hd, Wd, draft_dev, stream=side, **out)     # warm-up on the capture stream
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dmb.dropmatch_verify(runner.ctx, prm, hd, Wd, draft_dev, stream=torch.cuda.current_stream(), **out)
    seen = []
    for w in (0, 1, 5, 1):
        word.fill_(w)
        for v in out.values():
            v.fill_(7 if v.dtype == torch.uint8 else -1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = {k: v.cpu().numpy() for k, v in out.items()}
        eager = runner.verify(wl, hd, Wd, draft, seeds, step=(base + w) % 2 ** 32, **kw)   # eager work between replays
        for k in got:
            assert np.array_equal(got[k], eager[k]), f"word {w}: {k}"
        seen.append(got["path_ids"])
    assert (seen[0] != seen[1]).any() and (seen[1] != seen[2]).any() and np.array_equal(seen[1], seen[3])
    # the masks themselves, through the debug call: base + word, modulo 2^32
    word.fill_(3)
    bits = torch.zeros((wl.B, wl.T, wl.K, (wl.d + 31) // 32), dtype=torch.int32, device="cuda")
    dmb.dm_debug_masks(runner.ctx, prm, bits)
    torch.cuda.synchronize()
    want = np.stack([orc.pack_mask_bits(orc.keep_masks(int(s), (base + 3) % 2 ** 32, wl.T, wl.K, wl.d, wl.p)) for s in seeds])
    assert np.array_equal(bits.cpu().numpy().view(np.uint32), want)
    del graph, keep


# ------------------------------------------------------------------ clean last path
@pytest.mark.parametrize("d,V,B,T,K,dtype", [
    (256, 3000, 2, 6, 16, "bf16"),    # MFMA kernel, 192 rows -> 256-row tiles
    (256, 3000, 1, 8, 16, "bf16"),    # 128 rows: the W-streaming kernel
    (100, 130, 2, 3, 5, "f32"),       # generic kernel
])
def test_clean_last_path(runner, d, V, B, T, K, dtype):
    """Path K-1 without dropout: its token is the greedy token, its mask is all ones, its debug logits
    carry no 1/(1-p), and the rules see paths 0..K-2 only (oracle with the same option)."""
    wl, W, h, seeds, draft = _problem("clean", d, V, dtype, B, T, K, 0.3, seed=d + K, bonus=True)
    hd, Wd = to_device(h, dtype), to_device(W, dtype)
    flag = dmb.DM_FLAG_CLEAN_LAST_PATH
    for rule in (orc.RULE_ANY, orc.RULE_MAJORITY):
        ref = orc.verify(h, W, draft, seeds, K, wl.p, rule=rule, clean_last_path=True)
        res = runner.verify(wl, hd, Wd, draft, seeds, rule=rule, flags=flag)
        _check_against_oracle(res, ref, draft, rule, label=f"clean {dtype} M={B*T*K} rule={rule}")
        assert np.array_equal(res["path_ids"][:, :, -1], orc.greedy_ids(h, W))
        fewer = runner.verify(wl.with_(K=K - 1), hd, Wd, draft, seeds, rule=rule, K=K - 1)
        for k in ("vote_ids", "vote_cnt", "hit", "accept_len"):
            assert np.array_equal(res[k], fewer[k]), k
    bits = runner.masks(wl, seeds, flags=flag)
    plain = runner.masks(wl, seeds)
    nw = (d + 31) // 32
    full = np.full(nw, 0xFFFFFFFF, dtype=np.uint32)
    if d % 32:
        full[-1] = (1 << (d % 32)) - 1
    assert np.array_equal(bits[:, :, -1], np.broadcast_to(full, bits[:, :, -1].shape))
    assert np.array_equal(bits[:, :, :-1], plain[:, :, :-1])
    ref = orc.verify(h, W, draft, seeds, K, wl.p, clean_last_path=True, want_logits=(0, min(V, 200)))
    lg = runner.logits(wl, hd, Wd, seeds, 0, min(V, 200), flags=flag)
    assert np.abs(lg - ref["logits"]).max() < (2e-2 if dtype == "bf16" else 1e-3)


# ------------------------------------------------------------------ acceptance step inside the contraction launch
@pytest.mark.parametrize("B,T,K,tree", [(1, 8, 16, False), (2, 4, 16, False), (8, 2, 8, False), (1, 5, 5, False),
                                        (2, 16, 4, True)])
def test_fused_and_separate_acceptance_step_agree(runner, B, T, K, tree):
    """At most 128 masked rows, bf16: the vote / rule / prefix step runs in the workgroup of the
    contraction kernel that finishes last.  Same outputs as with the step as its own kernel, and as
    the oracle; repeated calls reuse the counter that elects that workgroup."""
    wl, W, h, seeds, draft = _problem("fuse", 256, 3000, "bf16", B, T, K, 0.2, seed=40 + B * T + K, bonus=not tree)
    parent = None
    if tree:
        parent = wk.make_tree_parents(wl.with_(tree=True), max_depth=5, max_branch=3)
        draft = wk.make_tree_draft_ids(wl, parent, orc.greedy_ids(h, W))
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    for rule in (orc.RULE_ANY, orc.RULE_MAJORITY):
        ref = orc.verify(h, W, draft, seeds, K, wl.p, rule=rule, parent=parent)
        for rep in range(3):
            fused = runner.verify(wl, hd, Wd, draft, seeds, rule=rule, parent=parent)
            _check_against_oracle(fused, ref, draft, rule, parent=parent, label=f"fused B={B} T={T} K={K} rule={rule}")
        apart = runner.verify(wl, hd, Wd, draft, seeds, rule=rule, parent=parent, flags=dmb.DM_FLAG_SEPARATE_VOTE)
        for k in fused:
            assert np.array_equal(fused[k], apart[k]), k


# ------------------------------------------------------------------ peaked heads (the regime of a real LM)
def test_planted_dominant_tokens(runner):
    """Hidden states with a planted dominant token (stand-in for the paper's agreement table, where all
    K = 5 paths agree at 98 % of positions): most rows are unanimous, drafts equal to the planted
    token are accepted under both rules, and everything matches the oracle."""
    wl = wk.Workload("planted", d=256, V=4096, dtype="bf16", B=4, T=8, K=5, p=0.3, bonus=True, data_seed=88)
    W = wk.make_weight(wl, sigma=0.05)
    h, planted = wk.make_planted_hidden(wl, W, alpha=14.0)
    seeds = wk.make_seeds(wl, base_seed=3)
    draft = planted.copy()
    draft[:, -1] = -1
    draft[1, 3] = (planted[1, 3] + 1) % wl.V          # one wrong draft token: the prefix stops there
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    for rule in (orc.RULE_ANY, orc.RULE_MAJORITY):
        ref = orc.verify(h, W, draft, seeds, wl.K, wl.p, rule=rule)
        res = runner.verify(wl, hd, Wd, draft, seeds, rule=rule)
        _check_against_oracle(res, ref, draft, rule, label=f"planted rule={rule}")
        assert (res["vote_cnt"] == wl.K).mean() > 0.9
        assert res["accept_len"].tolist() == [7, 3, 7, 7]


# ------------------------------------------------------------------ sampled path tokens
@pytest.mark.parametrize("d,V,B,T,K,dtype,tau", [
    (256, 3000, 1, 8, 16, "bf16", 1.0),    # W-streaming kernel, ragged last vocabulary tile
    (256, 4096, 2, 6, 16, "bf16", 0.7),    # 256 x 256 tiles
    (100, 130, 2, 3, 5, "f32", 1.5),       # generic kernel
    (128, 777, 1, 3, 16, "bf16", 0.25),    # a sharp temperature
    (1024, 2000, 2, 6, 16, "bf16", 0.7),   # 256 x 256 tiles of 16 slabs: noise drawn by the copy wavefronts; 192 of 256 rows
    (2048, 3000, 3, 7, 16, "bf16", 1.2),   # two row tiles (336 rows), ragged vocabulary, 32 slabs
    (1088, 600, 2, 5, 32, "bf16", 0.5),    # 17 slabs, K = 32, three vocabulary tiles
    (2112, 1500, 1, 8, 16, "bf16", 0.9),   # W-streaming kernel at 128 rows (noise drawn in its epilogue), 33 slabs, ragged tiles
    (1600, 1100, 1, 6, 16, "bf16", 1.1),   # the same at 96 rows, 25 slabs
    (4096, 700, 1, 7, 16, "bf16", 0.8),    # 112 of 128 rows at the benchmark's d
])
def test_sampled_path_tokens(runner, d, V, B, T, K, dtype, tau):
    """Path tokens drawn from Softmax(l / tau) by the Gumbel-max construction with the counter-based
    stream: equal to the oracle's draws except where the oracle's perturbed top-2 gap is inside the
    floating-point band (the logit error 1e-5 is divided by tau, so the band is 1e-3 * max(1, 1/tau))."""
    wl, W, h, seeds, draft = _problem("samp", d, V, dtype, B, T, K, 0.2, seed=d + V + K, bonus=True)
    hd, Wd = to_device(h, dtype), to_device(W, dtype)
    flag = dmb.DM_FLAG_SAMPLE_PATHS
    tol = 1e-3 * max(1.0, 1.0 / tau)
    for rule, step in ((orc.RULE_ANY, 0), (orc.RULE_MAJORITY, 5)):
        ref = orc.verify(h, W, draft, seeds, K, wl.p, rule=rule, step=step, temperature=tau)
        res = runner.verify(wl, hd, Wd, draft, seeds, rule=rule, step=step, flags=flag, temperature=tau)
        nflip, _ = compare_path_ids(res["path_ids"], ref, tol=tol, label=f"sampled {dtype} M={B*T*K} tau={tau}")
        exp = ref if nflip == 0 else orc.acceptance_from_path_ids(res["path_ids"], draft, rule)
        for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
            assert np.array_equal(res[k], exp[k]), k
    plain = runner.verify(wl, hd, Wd, draft, seeds)
    assert (plain["path_ids"] != res["path_ids"]).any()            # it does sample
    again = runner.verify(wl, hd, Wd, draft, seeds, rule=orc.RULE_MAJORITY, step=5, flags=flag, temperature=tau)
    assert np.array_equal(again["path_ids"], res["path_ids"])       # and is a pure function of its key
    # with a clean last path that path stays the greedy token
    both = runner.verify(wl, hd, Wd, draft, seeds, flags=flag | dmb.DM_FLAG_CLEAN_LAST_PATH, temperature=tau)
    assert np.array_equal(both["path_ids"][:, :, -1], orc.greedy_ids(h, W))
    refc = orc.verify(h, W, draft, seeds, K, wl.p, temperature=tau, clean_last_path=True)
    compare_path_ids(both["path_ids"], refc, tol=tol, label="sampled + clean last path")


def test_sampling_frequencies_on_the_gpu(runner):
    """Many steps on one small row: the GPU's own draws follow Softmax(l / tau) (chi-square against the
    distribution computed from the kernel's debug logits)."""
    import scipy.special
    import scipy.stats
    wl, W, h, seeds, draft = _problem("freq", 64, 12, "bf16", 1, 1, 64, 0.0, seed=17)
    hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
    tau = 0.05                                     # logits of this problem are small: sharpen them
    logits = runner.logits(wl, hd, Wd, seeds, 0, wl.V)[0].astype(np.float64)      # p = 0: every path alike
    want = scipy.special.softmax(logits / tau)
    counts = np.zeros(wl.V)
    for step in range(150):
        ids = runner.verify(wl, hd, Wd, draft, seeds, step=step, flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau)["path_ids"]
        counts += np.bincount(ids.reshape(-1), minlength=wl.V)
    keep = want * counts.sum() >= 5                 # chi-square needs expected counts of a few at least
    obs, expct = counts[keep], want[keep] * counts.sum()
    pval = scipy.stats.chisquare(obs, expct * obs.sum() / expct.sum())[1]
    assert pval > 1e-3, (counts, want * counts.sum())


# ------------------------------------------------------------------ measurement aid
@pytest.mark.parametrize("d,V,B,T,K,dtype", [
    (256, 1024, 1, 4, 16, "bf16"),    # W-streaming kernel (64 rows)
    (256, 1024, 2, 10, 16, "bf16"),   # 256 x 256 tiles (320 rows)
    (100, 130, 2, 3, 5, "f32"),       # generic kernel
])
def test_profiling_modes_time_kernels_and_leave_results_alone(runner, d, V, B, T, K, dtype):
    """dm_set_profiling: mode 2 times the contraction launch itself on every stride-th call, mode 1
    brackets every kernel; neither may change a result (mode 2 launches through another runtime call)."""
    wl, W, h, seeds, draft = _problem("prof", d, V, dtype, B, T, K, 0.1, seed=d + V + B, bonus=False)
    hd, Wd = to_device(h, dtype), to_device(W, dtype)
    plain = runner.verify(wl, hd, Wd, draft, seeds)
    try:
        dmb.dm_set_profiling_stride(runner.ctx, 3)
        dmb.dm_set_profiling(runner.ctx, 2)
        for _ in range(7):
            res = runner.verify(wl, hd, Wd, draft, seeds)
            for k in plain:
                assert np.array_equal(res[k], plain[k]), k
        n, ms = dmb.dm_get_profile_stages(runner.ctx)
        assert n == 3                                   # calls 0, 3 and 6
        assert 0.0 < ms[1] < 50.0 and ms[0] == 0.0 and ms[4] == 0.0
        samples = dmb.dm_get_profile_samples(runner.ctx, 1)        # the durations behind that mean
        assert len(samples) == 3 and all(x > 0.0 for x in samples) and np.mean(samples) == pytest.approx(ms[1], rel=1e-5)
        assert dmb.dm_get_profile_samples(runner.ctx, 0) == [] and dmb.dm_get_profile_samples(runner.ctx, 1, n_max=2) == samples[:2]

        dmb.dm_set_profiling_stride(runner.ctx, 1)
        dmb.dm_set_profiling(runner.ctx, 1)
        for _ in range(4):
            res = runner.verify(wl, hd, Wd, draft, seeds)
            for k in plain:
                assert np.array_equal(res[k], plain[k]), k
        n, ms = dmb.dm_get_profile_stages(runner.ctx)
        assert n == 4 and ms[0] > 0.0 and ms[1] > 0.0 and ms[4] >= 0.0 and ms[2] == 0.0 and ms[3] == 0.0  # no JS passes in dropmatch_verify
        n3, m0, m1, m4 = dmb.dm_get_profile(runner.ctx)
        assert n3 == 4 and m1 == pytest.approx(ms[1])
        assert len(dmb.dm_get_profile_samples(runner.ctx, 0)) == 4 and dmb.dm_get_profile_samples(runner.ctx, 2) == []
        with pytest.raises(dmb.DropMatchError):
            dmb.dm_get_profile_samples(runner.ctx, 5)

        dmb.dm_set_profiling(runner.ctx, 0)
        assert dmb.dm_get_profile_stages(runner.ctx)[0] == 0
        with pytest.raises(dmb.DropMatchError):
            dmb.dm_set_profiling_stride(runner.ctx, 0)
    finally:
        dmb.dm_set_profiling(runner.ctx, 0)
        dmb.dm_set_profiling_stride(runner.ctx, 1)


def test_stream_read_aid_and_its_argument_checks(runner):
    """dm_debug_stream_read enqueues a bare read of a buffer (the ceiling bench.py quotes beside the published
    HBM peak): it must leave the buffer alone, and refuse sizes and addresses that are not multiples of 16."""
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    before = buf.clone()
    for nbytes in (16, 4 << 20, (4 << 20) - 16):
        dmb.dm_debug_stream_read(runner.ctx, buf, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(buf, before)
    for bad in (0, 8, 24, -16):
        with pytest.raises(dmb.DropMatchError) as e:
            dmb.dm_debug_stream_read(runner.ctx, buf, bad)
        assert e.value.status == dmb.DM_EINVAL
    with pytest.raises(dmb.DropMatchError):
        dmb.dm_debug_stream_read(runner.ctx, buf[1:], 64)            # 4 bytes past a 16-byte boundary
