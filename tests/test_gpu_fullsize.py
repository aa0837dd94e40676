"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

head8b is checked in full against the oracle.  For the larger configurations the oracle
computes one position of every 256-row tile of masked rows (all K paths over the full
vocabulary, so every vocabulary tile including the ragged last one, every row tile, every
XCD patch and every round of the tile walk is compared), and every acceptance output is
checked bit-exactly against the oracle's vote/accept logic applied to the GPU's path
tokens (a property that holds at any size)."""
import gc

import numpy as np
import pytest

from oracle import dropmatch_oracle as orc
from paper_2603_03333_amd import workloads as wk

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2603_03333_amd import binding as dmb  # noqa: E402
from gpu_harness import Runner, compare_path_ids, to_device  # noqa: E402


NEAR_TOL = 1e-2


def _oracle_position(h, W64, seed, t, K, p):
    """Path tokens, top-2 gaps and near-tie candidates of the K paths of one row, by the oracle's own
    functions, in the form compare_path_ids takes.  Also returns the logits [K, V]."""
    d = h.shape[-1]
    Hm = np.stack([orc.masked_state(h, orc.keep_mask(int(seed), 0, t, i, d, p), p) for i in range(K)])
    L = (W64 @ Hm.T).T
    toks = [orc.path_token(L[i]) for i in range(K)]
    ref = dict(path_ids=np.array([x[0] for x in toks], dtype=np.int32), gap=np.array([x[1] for x in toks]),
               near={(i,): orc.tokens_within(L[i], NEAR_TOL) for i in range(K) if toks[i][1] <= NEAR_TOL},
               near_tol=NEAR_TOL)
    return ref, L


def _one_position_per_row_tile(wl, stride=1):
    """(b, t) of one position inside every `stride`-th 256-row tile of masked rows (rows are ordered
    (b, t, path)), first and last tile always included, at a place inside the tile that moves from tile
    to tile."""
    per_tile = max(1, 256 // wl.K)                       # positions per row tile
    n_pos = wl.B * wl.T
    n_tiles = (wl.rows + 255) // 256
    tiles = sorted(set(range(0, n_tiles, stride)) | {n_tiles - 1})
    out = []
    for j in tiles:
        pos = min(j * per_tile + (5 * j + 3) % per_tile, n_pos - 1)
        out.append((pos // wl.T, pos % wl.T))
    return out


def _run_config(name, sample, wl=None):
    wl = wl or wk.CONFIGS[name]
    print(f"[{name}] generating inputs", flush=True)
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl)
    W64 = W.astype(np.float64)
    greedy = np.zeros((wl.B, wl.T), dtype=np.int32)      # plant greedy tokens only at the sampled rows
    parent = wk.make_tree_parents(wl) if wl.tree else None
    rows = _one_position_per_row_tile(wl) if sample else [(b, t) for b in range(wl.B) for t in range(wl.T)]
    for b, t in rows:
        greedy[b, t] = orc.path_token(W64 @ h[b, t].astype(np.float64))[0]
    draft = wk.make_tree_draft_ids(wl, parent, greedy) if wl.tree else wk.make_draft_ids(wl, greedy)

    r = Runner(wl.rows, wl.d, wl.V)
    try:
        prm, _ = r.params(wl, seeds)
        assert dmb.dm_kernel_choice(prm) == 1
        hd, Wd = to_device(h, wl.dtype), to_device(W, wl.dtype)
        print(f"[{name}] running the HIP path", flush=True)
        res = r.verify(wl, hd, Wd, draft, seeds, parent=parent)
        # repeated calls (for at most 128 rows the acceptance step runs inside the contraction launch,
        # elected by a counter that every call has to leave at zero): identical outputs every time
        for rep in range(40 if wl.rows <= 128 else 1):
            res2 = r.verify(wl, hd, Wd, draft, seeds, parent=parent)
            for k in res:
                assert np.array_equal(res[k], res2[k]), f"{k} not deterministic (repetition {rep})"
        # masks of sampled rows, bit-exact
        bits = r.masks(wl, seeds)
        for b, t in rows[:4]:
            want = orc.pack_mask_bits(np.stack([orc.keep_mask(int(seeds[b]), 0, t, i, wl.d, wl.p) for i in range(wl.K)]))
            assert np.array_equal(bits[b, t], want)
        del hd, Wd
    finally:
        r.close()
    torch.cuda.empty_cache()

    print(f"[{name}] oracle on {len(rows)} positions", flush=True)
    ndiff = nnear = 0
    for b, t in rows:
        ref, _ = _oracle_position(h[b, t], W64, seeds[b], t, wl.K, wl.p)
        a, c = compare_path_ids(res["path_ids"][b, t], ref)
        ndiff += a
        nnear += c
    print(f"[{name}] checked positions={len(rows)} (one per 256-row tile) rows={len(rows) * wl.K} "
          f"near-tie rows(gap<1e-3)={nnear} path-token flips={ndiff}", flush=True)
    # vote / rule / prefix-or-tree logic on the GPU's own path tokens: exact at any size
    expect = orc.acceptance_from_path_ids(res["path_ids"], draft, orc.RULE_ANY, parent)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], expect[k]), f"{name}: {k} differs"
    assert (res["path_ids"] >= 0).all() and (res["path_ids"] < wl.V).all()
    del W, W64
    gc.collect()
    return res


def test_head8b_full():
    res = _run_config("head8b", sample=0)
    assert res["accept_len"].shape == (1,) and 0 <= res["accept_len"][0] <= 7    # bonus row never hits


def test_bigvocab_one_position_per_row_tile():
    _run_config("bigvocab", sample=True)


def test_tree_one_position_per_row_tile():
    res = _run_config("tree", sample=True)
    assert (res["accept_len"] <= 6).all() and (res["hit"][:, 0] == 1).all()


def test_batched_one_position_per_row_tile():
    _run_config("batched", sample=True)


@pytest.mark.parametrize("B", [2, 4])
def test_head8b_shape_between_the_two_kernels(B):
    """256 and 512 masked rows at the head8b shape: the points of the rows sweep where W still streams from memory
    but the 256 x 256 kernel runs (one or two row tiles, two or four rounds of vocabulary tiles per workgroup).
    Every position against the oracle."""
    wl = wk.CONFIGS["head8b"].with_(B=B, data_seed=1010 + B)
    _run_config(f"head8b-shape B={B}", sample=False, wl=wl)


# ------------------------------------------------------------------ distribution-level rule (Eq. 5, 6, Alg. 1)
def _run_config_js(name, sample):
    from gpu_harness import JS_ATOL, JS_RTOL
    wl = wk.CONFIGS[name]
    print(f"[{name}/js] generating inputs", flush=True)
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl)
    hd, Wd = to_device(h, wl.dtype), to_device(W, wl.dtype)
    # undropped head logits for the draft stand-in: a plain library matmul, input preparation only
    clean = (hd.float().reshape(-1, wl.d) @ Wd.float().T).reshape(wl.B, wl.T, wl.V).cpu().numpy()
    greedy = clean.argmax(-1).astype(np.int32)
    draft = wk.make_draft_ids(wl, greedy)
    probs = wk.make_draft_probs(wl, clean)
    del clean
    r = Runner(wl.rows, wl.d, wl.V)
    try:
        r.reserve_js(wl.B * wl.T, wl.K)
        print(f"[{name}/js] running the HIP path", flush=True)
        res = r.verify_js(wl, hd, Wd, draft, probs, seeds, rule=dmb.DM_RULE_JS_OR_MAJORITY)
        res2 = r.verify_js(wl, hd, Wd, draft, probs, seeds, rule=dmb.DM_RULE_JS_OR_MAJORITY)
        for k in res:
            assert np.array_equal(res[k], res2[k], equal_nan=True), f"{k} not deterministic"
        del hd, Wd
    finally:
        r.close()
    torch.cuda.empty_cache()

    W64 = W.astype(np.float64)
    rows = _one_position_per_row_tile(wl) if sample else [(b, t) for b in range(wl.B) for t in range(wl.T)]
    print(f"[{name}/js] oracle on {len(rows)} positions", flush=True)
    near = nflip = ntie = 0
    worst_h = worst_d = 0.0
    for b, t in rows:
        ref, L = _oracle_position(h[b, t], W64, seeds[b], t, wl.K, wl.p)
        a, c = compare_path_ids(res["path_ids"][b, t], ref)
        nflip += a
        ntie += c
        js_hit, jd, jh = orc.js_rule(probs[b, t], L)
        assert np.all(np.abs(res["js_heads"][b, t] - jh) <= JS_ATOL + JS_RTOL * np.abs(jh)), (b, t)
        worst_h = max(worst_h, float(np.abs(res["js_heads"][b, t] - jh).max()))
        if draft[b, t] < 0:
            assert res["js_draft"][b, t] == -1.0 and res["hit"][b, t] == 0
            continue
        assert abs(res["js_draft"][b, t] - jd) <= JS_ATOL + JS_RTOL * abs(jd), (b, t)
        worst_d = max(worst_d, abs(float(res["js_draft"][b, t]) - jd))
        if abs(jh.max() - jd) <= 2 * (JS_ATOL + JS_RTOL * abs(jd)):
            near += 1
        else:
            gpu_js = res["js_draft"][b, t] <= res["js_heads"][b, t].max()
            assert bool(gpu_js) == bool(js_hit), (b, t)
    print(f"[{name}/js] checked positions={len(rows)} Eq. (6) near-tie={near} max|d js_heads|={worst_h:.2e} "
          f"max|d js_draft|={worst_d:.2e} path tokens: near-tie rows={ntie} flips={nflip}", flush=True)
    # rule + prefix logic on the GPU's own JS values and path tokens: exact at any size
    has = draft >= 0
    gpu_js = has & (res["js_draft"] <= res["js_heads"].max(-1))
    votes = orc.acceptance_from_path_ids(res["path_ids"], draft, orc.RULE_MAJORITY)
    want = gpu_js | votes["hit"].astype(bool)
    assert np.array_equal(res["hit"].astype(bool), want)
    exp = orc.acceptance_from_hits(want)
    for k in ("accept_mask", "accept_len", "best_node"):
        assert np.array_equal(res[k], exp[k]), f"{name}/js: {k} differs"
    assert np.array_equal(res["vote_ids"], votes["vote_ids"])
    del W, W64
    gc.collect()


def test_head8b_js_full():
    _run_config_js("head8b", sample=0)


def test_batched_js_one_position_per_row_tile():
    _run_config_js("batched", sample=True)


# ------------------------------------------------------------------ sampled path tokens at full size
def _check_sampled(gpu_tok, logits, tau, g, where, tol=1.25e-3):
    """One sampled path token against the oracle's draw: equal, or (perturbed top-2 gap below tol) one of
    the tokens whose perturbed value is within tol of the maximum.  Returns (near-tie?, differs?)."""
    y, gap = orc.sampled_token(logits, tau, g)
    if gpu_tok == y:
        return int(gap < tol), 0
    assert gap < tol, (where, gap)
    ids, _ = orc.tokens_within(orc.sampled_values(logits, tau, g), tol)
    assert int(gpu_tok) in ids, (where, int(gpu_tok), ids.tolist())
    return 1, 1


@pytest.mark.parametrize("K", [16, 5])     # 128 rows: noise drawn in the epilogue; 40 rows: added during the k loop
def test_head8b_sampled_tokens_on_sampled_rows(K):
    wl = wk.CONFIGS["head8b"].with_(K=K)
    tau = 0.8
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl)
    draft = wk.make_draft_ids(wl, None)
    r = Runner(wl.rows, wl.d, wl.V)
    try:
        hd, Wd = to_device(h, wl.dtype), to_device(W, wl.dtype)
        res = r.verify(wl, hd, Wd, draft, seeds, flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau)
        res2 = r.verify(wl, hd, Wd, draft, seeds, flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau)
        assert np.array_equal(res["path_ids"], res2["path_ids"])
        del hd, Wd
    finally:
        r.close()
    torch.cuda.empty_cache()
    W64 = W.astype(np.float64)
    near = flips = 0
    for t in (0, 5):                                    # two positions, all K paths each, full vocabulary
        Hm = np.stack([orc.masked_state(h[0, t], orc.keep_mask(int(seeds[0]), 0, t, i, wl.d, wl.p), wl.p)
                       for i in range(wl.K)])
        L = W64 @ Hm.T
        for i in range(wl.K):
            g = orc.gumbel_noise(orc.sampling_uniforms(int(seeds[0]), 0, t, i, wl.V))
            n, f = _check_sampled(res["path_ids"][0, t, i], L[:, i], tau, g, (t, i))
            near += n
            flips += f
    print(f"[head8b/sampled K={K}] rows={2 * K} near-tie={near} flips={flips}", flush=True)
    exp = orc.acceptance_from_path_ids(res["path_ids"], draft, orc.RULE_ANY)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_len"):
        assert np.array_equal(res[k], exp[k]), k


def test_head8b_nucleus_tokens_on_sampled_rows():
    """Top-p draws at the full head8b size (126 chunks of vocabulary rows per position in the launch
    configuration bench.py times): two positions, all 16 paths, checked as in test_gpu_nucleus.py."""
    from test_gpu_nucleus import check_nucleus_tokens
    wl = wk.CONFIGS["head8b"]
    tau, top_p = 0.8, 0.9
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl)
    draft = wk.make_draft_ids(wl, None)
    r = Runner(wl.rows, wl.d, wl.V)
    try:
        r.reserve_js(wl.B * wl.T, wl.K)
        hd, Wd = to_device(h, wl.dtype), to_device(W, wl.dtype)
        kw = dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau, top_p=top_p)
        res = r.verify(wl, hd, Wd, draft, seeds, **kw)
        res2 = r.verify(wl, hd, Wd, draft, seeds, **kw)
        assert np.array_equal(res["path_ids"], res2["path_ids"])
        free = r.verify(wl, hd, Wd, draft, seeds, flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau)
        del hd, Wd
    finally:
        r.close()
    torch.cuda.empty_cache()
    W64 = W.astype(np.float64)
    rows = same = 0
    for t in (1, 6):
        Hm = np.stack([orc.masked_state(h[0, t], orc.keep_mask(int(seeds[0]), 0, t, i, wl.d, wl.p), wl.p)
                       for i in range(wl.K)])
        L = (W64 @ Hm.T).T                                # [K, V]
        # check_nucleus_tokens indexes logits by (b*T + t)*K + i: give it a one-position problem
        n, s = check_nucleus_tokens(res["path_ids"][:, t:t + 1], L, [int(seeds[0])], 0, tau, top_p, 1, 1, wl.K, wl.K, t0=t)
        rows += n
        same += s
    print(f"[head8b/nucleus] rows={rows} equal to the oracle's draw={same} "
          f"differ from the unrestricted draw={(res['path_ids'] != free['path_ids']).sum()} of {res['path_ids'].size}", flush=True)
    assert same >= 0.9 * rows
    exp = orc.acceptance_from_path_ids(res["path_ids"], draft, orc.RULE_ANY)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_len"):
        assert np.array_equal(res[k], exp[k]), k


def test_batched_sampled_tokens_on_sampled_rows():
    """Sampled path tokens at the full size of the compute-bound configuration (4096 rows, d = 8192:
    the 256 x 256 kernel whose copy wavefronts draw the noise, 31 tiles per workgroup): three positions
    from different sequences and row tiles, all 16 paths each over the full vocabulary."""
    wl = wk.CONFIGS["batched"]
    tau = 0.8
    W, h, seeds = wk.make_weight(wl), wk.make_hidden(wl), wk.make_seeds(wl)
    draft = wk.make_draft_ids(wl, None)
    r = Runner(wl.rows, wl.d, wl.V)
    try:
        hd, Wd = to_device(h, wl.dtype), to_device(W, wl.dtype)
        res = r.verify(wl, hd, Wd, draft, seeds, flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau)
        res2 = r.verify(wl, hd, Wd, draft, seeds, flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=tau)
        assert np.array_equal(res["path_ids"], res2["path_ids"])
        del hd, Wd
    finally:
        r.close()
    torch.cuda.empty_cache()
    near = flips = 0
    chunk = 16384                                       # vocabulary rows per float64 block of W
    for b, t in ((0, 0), (13, 3), (wl.B - 1, wl.T - 1)):
        Hm = np.stack([orc.masked_state(h[b, t], orc.keep_mask(int(seeds[b]), 0, t, i, wl.d, wl.p), wl.p)
                       for i in range(wl.K)])
        L = np.concatenate([W[v:v + chunk].astype(np.float64) @ Hm.T for v in range(0, wl.V, chunk)])
        for i in range(wl.K):
            g = orc.gumbel_noise(orc.sampling_uniforms(int(seeds[b]), 0, t, i, wl.V))
            n, f = _check_sampled(res["path_ids"][b, t, i], L[:, i], tau, g, (b, t, i))
            near += n
            flips += f
        del L
        gc.collect()
    print(f"[batched/sampled] rows=48 near-tie={near} flips={flips}", flush=True)
    exp = orc.acceptance_from_path_ids(res["path_ids"], draft, orc.RULE_ANY)
    for k in ("vote_ids", "vote_cnt", "hit", "accept_len"):
        assert np.array_equal(res[k], exp[k]), k
