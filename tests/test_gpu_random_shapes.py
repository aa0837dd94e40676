"""Seeded random shapes and option combinations against the oracle: ragged vocabulary tails, row
counts around the tile edges of every kernel, both storage types, every token-level option.  Each
case is small enough for the oracle to run in well under a second."""
import numpy as np
import pytest

from oracle import dropmatch_oracle as orc
from paper_2603_03333_amd import workloads as wk

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2603_03333_amd import binding as dmb  # noqa: E402
from gpu_harness import Runner, compare_js, compare_path_ids, to_device  # noqa: E402


@pytest.fixture(scope="module")
def runner():
    r = Runner(max_rows=1024, max_d=512, max_V=4096)
    r.reserve_js(max_positions=64, max_K=64)
    yield r
    r.close()


def _draw(case):
    rng = np.random.default_rng(7000 + case)
    bf16 = rng.random() < 0.75
    d = int(rng.choice([64, 128, 192, 256, 512])) if (bf16 and rng.random() < 0.8) else int(rng.integers(5, 200))
    V = int(rng.choice([1, 7, 255, 256, 257, 511, 1000, 2049, 4096]) if rng.random() < 0.5 else rng.integers(2, 3000))
    K = int(rng.choice([1, 2, 3, 5, 8, 16, 17, 32, 40]))
    T = int(rng.integers(1, 10))
    B = int(rng.integers(1, 5))
    while B * T * K > 1024:
        T = max(1, T - 1)
        B = max(1, B - 1)
    p = float(rng.choice([0.0, 0.05, 0.1, 0.3, 0.5, 0.9]))
    return rng, ("bf16" if bf16 else "f32"), d, V, B, T, K, p


@pytest.mark.parametrize("case", range(48))
def test_random_token_level_case(runner, case):
    rng, dtype, d, V, B, T, K, p = _draw(case)
    wl = wk.Workload(f"rand{case}", d=d, V=V, dtype=dtype, B=B, T=T, K=K, p=p, bonus=bool(rng.integers(0, 2)),
                     data_seed=9000 + case)
    W, h = wk.make_weight(wl, sigma=0.1), wk.make_hidden(wl)
    seeds = rng.integers(0, 2 ** 63, size=B, dtype=np.uint64)
    step = int(rng.integers(0, 2 ** 32))
    rule = int(rng.integers(0, 2))
    share = bool(rng.integers(0, 2))
    clean = K >= 2 and rng.random() < 0.3
    tree = T >= 3 and rng.random() < 0.3
    tau = float(rng.choice([0.5, 1.0, 2.0])) if rng.random() < 0.3 else None
    greedy = orc.greedy_ids(h, W)
    parent = None
    if tree:
        parent = wk.make_tree_parents(wl.with_(tree=True), max_depth=4, max_branch=3)
        draft = wk.make_tree_draft_ids(wl, parent, greedy)
    else:
        draft = wk.make_draft_ids(wl, greedy)
    flags = (dmb.DM_FLAG_SHARE_MASK_ACROSS_POS if share else 0) | (dmb.DM_FLAG_CLEAN_LAST_PATH if clean else 0) | \
            (dmb.DM_FLAG_SAMPLE_PATHS if tau else 0) | (dmb.DM_FLAG_SEPARATE_VOTE if rng.random() < 0.3 else 0) | \
            (dmb.DM_FLAG_FORCE_GENERIC if rng.random() < 0.2 else 0)
    ref = orc.verify(h, W, draft, seeds, K, p, step=step, rule=rule, share_mask_across_pos=share, parent=parent,
                     clean_last_path=clean, temperature=tau)
    res = runner.verify(wl, to_device(h, dtype), to_device(W, dtype), draft, seeds, step=step, rule=rule, flags=flags,
                        parent=parent, temperature=tau or 0.0)
    tol = 1e-3 * (max(1.0, 1.0 / tau) if tau else 1.0)
    nflip, nnear = compare_path_ids(res["path_ids"], ref, tol=tol)
    KU = K - 1 if clean else K
    exp = ref if nflip == 0 else orc.acceptance_from_path_ids(res["path_ids"][:, :, :KU], draft, rule, parent)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], exp[k]), f"case {case} ({dtype} d={d} V={V} B={B} T={T} K={K} p={p} flags={flags}): {k}"


@pytest.mark.parametrize("case", range(16))
def test_random_js_case(runner, case):
    rng, dtype, d, V, B, T, K, p = _draw(100 + case)
    V = max(V, 2)
    while B * T > 64:
        B = max(1, B - 1)
    p = min(p, 0.5)
    wl = wk.Workload(f"randjs{case}", d=d, V=V, dtype=dtype, B=B, T=T, K=K, p=p, bonus=bool(rng.integers(0, 2)),
                     data_seed=9500 + case)
    W, h = wk.make_weight(wl, sigma=0.1), wk.make_hidden(wl)
    seeds = rng.integers(0, 2 ** 63, size=B, dtype=np.uint64)
    clean = K >= 2 and rng.random() < 0.3
    rule = int(rng.integers(2, 4))
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    clean_logits = np.einsum("vd,btd->btv", W.astype(np.float64), h.astype(np.float64)).astype(np.float32)
    probs = wk.make_draft_probs(wl, clean_logits, topk=int(rng.choice([0, 0, 5])) if V > 8 else 0)
    flags = dmb.DM_FLAG_CLEAN_LAST_PATH if clean else 0
    ref = orc.verify_js(h, W, draft, probs, seeds, K, p, rule=rule, clean_last_path=clean)
    res = runner.verify_js(wl, to_device(h, dtype), to_device(W, dtype), draft, probs, seeds, rule=rule, flags=flags)
    nflip, _ = compare_path_ids(res["path_ids"], ref)
    n_tie, gpu_js = compare_js(res, ref, draft, rule == 2, nflip, f"rand js {case} {dtype} d={d} V={V} B={B} T={T} K={K}")
    KU = K - 1 if clean else K
    votes = orc.acceptance_from_path_ids(res["path_ids"][:, :, :KU], draft, orc.RULE_MAJORITY)
    want = gpu_js | (votes["hit"].astype(bool) if rule == 3 else False)
    assert np.array_equal(res["hit"].astype(bool), want)
    assert np.array_equal(res["accept_len"], orc.acceptance_from_hits(want)["accept_len"])


@pytest.fixture(scope="module")
def medium_runner():
    r = Runner(max_rows=8192, max_d=512, max_V=70000)
    yield r
    r.close()


def _draw_medium(case):
    rng = np.random.default_rng(31000 + case)
    d = int(rng.choice([64, 128, 256, 512]))
    V = int(rng.integers(256, 66000)) if case % 4 else int(rng.choice([256, 257, 511, 512, 65536, 65537]))
    K = int(rng.choice([4, 8, 16, 32]))
    T = int(rng.integers(2, 17))
    B = int(rng.integers(1, 33))
    while B * T * K > 8192 or B * T * K * V > 6e7:   # keeps the oracle's float64 logits near 0.5 GB
        B = max(1, B // 2)
        if B == 1:
            T = max(1, T // 2)
        if B == 1 and T == 1:
            V = V // 2 + 256
    return rng, d, V, B, T, K


@pytest.mark.parametrize("case", [0, 3, 4, 7, 9, 12, 16, 18, 26, 27, 28, 36])
def test_random_medium_case(medium_runner, case):
    """Several row blocks times hundreds of vocabulary tiles (the persistent tile walk of the 256 x 256
    kernel, ragged in both directions), every path token against the oracle; every fifth case samples."""
    rng, d, V, B, T, K = _draw_medium(case)
    wl = wk.Workload(f"med{case}", d=d, V=V, dtype="bf16", B=B, T=T, K=K, p=0.1, bonus=False, data_seed=12000 + case)
    W, h = wk.make_weight(wl, sigma=0.1), wk.make_hidden(wl)
    seeds = rng.integers(0, 2 ** 63, size=B, dtype=np.uint64)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    tau = 1.0 if case % 5 == 0 else None
    rule = case % 2
    ref = orc.verify(h, W, draft, seeds, K, 0.1, rule=rule, temperature=tau)
    res = medium_runner.verify(wl, to_device(h, "bf16"), to_device(W, "bf16"), draft, seeds, rule=rule,
                               flags=dmb.DM_FLAG_SAMPLE_PATHS if tau else 0, temperature=tau or 0.0)
    nflip, nnear = compare_path_ids(res["path_ids"], ref)
    print(f"[medium {case}: d={d} V={V} B={B} T={T} K={K} rows={B*T*K} tau={tau}] near-tie rows={nnear} flips={nflip}", flush=True)
    exp = ref if nflip == 0 else orc.acceptance_from_path_ids(res["path_ids"], draft, rule, None)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], exp[k]), f"medium case {case}: {k}"


def test_sampled_tokens_over_several_tiles_per_workgroup():
    """Sampled path tokens where every workgroup of the 256 x 256 kernel walks two or three tiles
    (548 tiles on 256 compute units) of 16 slabs each: the copy wavefronts draw a tile's noise while
    the tile before is still being reduced.  Every path token against the oracle; one sequence has
    a clean last path."""
    import gc
    d, V, B, T, K, tau = 1024, 70000, 4, 8, 16, 0.9
    wl = wk.Workload("samp_multi", d=d, V=V, dtype="bf16", B=B, T=T, K=K, p=0.1, bonus=True, data_seed=4242)
    W, h = wk.make_weight(wl, sigma=0.1), wk.make_hidden(wl)
    seeds = np.random.default_rng(99).integers(0, 2 ** 63, size=B, dtype=np.uint64)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    r = Runner(max_rows=B * T * K, max_d=d, max_V=V)
    try:
        hd, Wd = to_device(h, "bf16"), to_device(W, "bf16")
        for clean in (False, True):
            flags = dmb.DM_FLAG_SAMPLE_PATHS | (dmb.DM_FLAG_CLEAN_LAST_PATH if clean else 0)
            res = r.verify(wl, hd, Wd, draft, seeds, rule=1, step=3, flags=flags, temperature=tau)
            ref = orc.verify(h, W, draft, seeds, K, 0.1, rule=1, step=3, temperature=tau, clean_last_path=clean)
            nflip, nnear = compare_path_ids(res["path_ids"], ref, tol=1e-3 / tau)
            print(f"[sampled, several tiles per workgroup, clean={clean}] rows={B*T*K} near-tie rows={nnear} flips={nflip}", flush=True)
            KU = K - 1 if clean else K
            exp = ref if nflip == 0 else orc.acceptance_from_path_ids(res["path_ids"][:, :, :KU], draft, 1, None)
            for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
                assert np.array_equal(res[k], exp[k]), k
            if clean:
                assert np.array_equal(res["path_ids"][:, :, -1], orc.greedy_ids(h, W))
            del ref
            gc.collect()
    finally:
        r.close()


def _draw_sampled_big(case):
    rng = np.random.default_rng(52000 + case)
    d = int(rng.choice([1024, 1088, 1536, 2048, 3072]))
    V = int(rng.integers(300, 9000)) if case % 3 else int(rng.choice([256, 257, 512, 4096, 4097]))
    K = int(rng.choice([3, 5, 8, 16, 17, 32]))
    T = int(rng.integers(2, 9))
    B = int(rng.integers(1, 5))
    while B * T * K <= 128:                       # more than 128 rows: the 256 x 256 kernel
        T += 1
    while B * T * K > 1024:
        T = max(1, T - 1)
    return rng, d, V, B, T, K


@pytest.mark.parametrize("case", range(10))
def test_random_sampled_case_on_the_big_kernel(case):
    """Sampled path tokens on the 256 x 256 kernel with 16 to 48 slabs per tile (the copy wavefronts draw
    the noise): ragged row and vocabulary counts, path counts that do not divide a row tile, several
    seeds, both token rules, with and without the clean path; every path token against the oracle."""
    import gc
    rng, d, V, B, T, K = _draw_sampled_big(case)
    assert B * T * K > 128
    tau = float(rng.choice([0.5, 1.0, 2.0]))
    clean = K >= 2 and bool(rng.integers(0, 2))
    rule = int(rng.integers(0, 2))
    step = int(rng.integers(0, 2 ** 32))
    wl = wk.Workload(f"sbig{case}", d=d, V=V, dtype="bf16", B=B, T=T, K=K, p=float(rng.choice([0.05, 0.1, 0.3])),
                     bonus=bool(rng.integers(0, 2)), data_seed=15000 + case)
    W, h = wk.make_weight(wl, sigma=0.05), wk.make_hidden(wl)
    seeds = rng.integers(0, 2 ** 63, size=B, dtype=np.uint64)
    draft = wk.make_draft_ids(wl, orc.greedy_ids(h, W))
    flags = dmb.DM_FLAG_SAMPLE_PATHS | (dmb.DM_FLAG_CLEAN_LAST_PATH if clean else 0)
    ref = orc.verify(h, W, draft, seeds, K, wl.p, rule=rule, step=step, temperature=tau, clean_last_path=clean)
    r = Runner(max_rows=B * T * K, max_d=d, max_V=V)
    try:
        res = r.verify(wl, to_device(h, "bf16"), to_device(W, "bf16"), draft, seeds, rule=rule, step=step, flags=flags,
                       temperature=tau)
    finally:
        r.close()
    tol = 1e-3 * max(1.0, 1.0 / tau)
    nflip, nnear = compare_path_ids(res["path_ids"], ref, tol=tol)
    print(f"[sampled big {case}: d={d} V={V} B={B} T={T} K={K} rows={B*T*K} tau={tau} clean={clean}] near-tie rows={nnear} flips={nflip}", flush=True)
    KU = K - 1 if clean else K
    exp = ref if nflip == 0 else orc.acceptance_from_path_ids(res["path_ids"][:, :, :KU], draft, rule, None)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], exp[k]), f"case {case}: {k}"
    gc.collect()
