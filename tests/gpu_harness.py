"""Helpers shared by the GPU parity tests: upload a workload, call the C ABI through the
binding, bring results back as numpy."""
import numpy as np
import torch

from paper_2603_03333_amd import binding as dmb
from paper_2603_03333_amd import workloads as wk


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 host array (already holding values of the storage dtype) -> device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)      # exact: the values are bf16-representable
    return t.cuda()


GUARD = 64      # canary elements in front of and behind every output buffer


class Guarded:
    """Output tensors with canary elements on both sides: the library gets a pointer into the middle
    of a larger allocation, and check() fails if anything outside the tensor's own elements changed."""

    def __init__(self, device="cuda"):
        self.bufs = {}
        self.device = device

    def make(self, name, shape, dtype, fill):
        n = int(np.prod(shape))
        canary = 0xA5 if dtype == torch.uint8 else (float("-inf") if dtype.is_floating_point else -0x5EED5EED)
        buf = torch.full((n + 2 * GUARD,), canary, dtype=dtype, device=self.device)
        view = buf[GUARD:GUARD + n].view(shape)
        view.fill_(fill)
        self.bufs[name] = (buf, n, canary)
        return view

    def check(self):
        for name, (buf, n, canary) in self.bufs.items():
            edge = torch.cat([buf[:GUARD], buf[GUARD + n:]]).cpu().numpy()
            want = np.full(edge.shape, canary, dtype=edge.dtype)
            assert np.array_equal(edge, want), f"{name}: the library wrote outside the output buffer"


class Runner:
    """Owns a context sized for one workload shape."""

    def __init__(self, max_rows, max_d, max_V):
        self.ctx = dmb.dm_create(0, max_rows, max_d, max_V)

    def close(self):
        if self.ctx is not None:
            dmb.dm_destroy(self.ctx)
            self.ctx = None

    def params(self, wl, seeds, p=None, step=0, rule=dmb.DM_RULE_ANY, flags=0, parent=None, K=None, temperature=0.0,
               top_p=0.0):
        dtype = dmb.DM_BF16 if wl.dtype == "bf16" else dmb.DM_F32
        return dmb.make_params(wl.B, wl.T, wl.K if K is None else K, wl.d, wl.V, dtype,
                               wl.p if p is None else p, [int(s) for s in seeds], step=step, rule=rule,
                               flags=flags, parent=parent, temperature=temperature, top_p=top_p)

    def verify(self, wl, h_dev, W_dev, draft, seeds, parent=None, **kw):
        K = kw.get("K") or wl.K
        B, T = wl.B, wl.T
        dev = "cuda"
        par_dev = None if parent is None else torch.from_numpy(np.ascontiguousarray(parent, dtype=np.int32)).cuda()
        prm, keep = self.params(wl, seeds, parent=par_dev, **kw)
        draft_dev = torch.from_numpy(np.ascontiguousarray(draft, dtype=np.int32)).cuda()
        guard = Guarded()
        out = dict(
            accept_len=guard.make("accept_len", (B,), torch.int32, -7),
            best_node=guard.make("best_node", (B,), torch.int32, -7),
            accept_mask=guard.make("accept_mask", (B, T), torch.uint8, 9),
            hit=guard.make("hit", (B, T), torch.uint8, 9),
            path_ids=guard.make("path_ids", (B, T, K), torch.int32, -7),
            vote_ids=guard.make("vote_ids", (B, T), torch.int32, -7),
            vote_cnt=guard.make("vote_cnt", (B, T), torch.int32, -7),
        )
        dmb.dropmatch_verify(self.ctx, prm, h_dev, W_dev, draft_dev, **out)
        torch.cuda.synchronize()
        guard.check()
        del keep
        return {k: v.cpu().numpy() for k, v in out.items()}

    def reserve_js(self, max_positions, max_K):
        dmb.dm_reserve_js(self.ctx, max_positions, max_K)

    def verify_js(self, wl, h_dev, W_dev, draft, draft_probs, seeds, rule=dmb.DM_RULE_JS_OR_MAJORITY, **kw):
        """dropmatch_verify_js through the C ABI; draft_probs is a host float32 array [B,T,V]."""
        K = kw.get("K") or wl.K
        B, T = wl.B, wl.T
        dev = "cuda"
        prm, keep = self.params(wl, seeds, rule=rule, **kw)
        draft_dev = torch.from_numpy(np.ascontiguousarray(draft, dtype=np.int32)).cuda()
        probs_dev = torch.from_numpy(np.ascontiguousarray(draft_probs, dtype=np.float32)).cuda()
        guard = Guarded()
        out = dict(
            accept_len=guard.make("accept_len", (B,), torch.int32, -7),
            best_node=guard.make("best_node", (B,), torch.int32, -7),
            accept_mask=guard.make("accept_mask", (B, T), torch.uint8, 9),
            hit=guard.make("hit", (B, T), torch.uint8, 9),
            path_ids=guard.make("path_ids", (B, T, K), torch.int32, -7),
            vote_ids=guard.make("vote_ids", (B, T), torch.int32, -7),
            vote_cnt=guard.make("vote_cnt", (B, T), torch.int32, -7),
            js_draft=guard.make("js_draft", (B, T), torch.float32, float("nan")),
            js_heads=guard.make("js_heads", (B, T, K), torch.float32, float("nan")),
        )
        dmb.dropmatch_verify_js(self.ctx, prm, h_dev, W_dev, draft_dev, probs_dev, **out)
        torch.cuda.synchronize()
        guard.check()
        del keep
        return {k: v.cpu().numpy() for k, v in out.items()}

    def masks(self, wl, seeds, **kw):
        K = kw.get("K") or wl.K
        nw = (wl.d + 31) // 32
        prm, keep = self.params(wl, seeds, **kw)
        guard = Guarded()
        bits = guard.make("bits", (wl.B, wl.T, K, nw), torch.int32, 0x5A5A5A5A)
        dmb.dm_debug_masks(self.ctx, prm, bits)
        torch.cuda.synchronize()
        guard.check()
        return bits.cpu().numpy().view(np.uint32)

    def logits(self, wl, h_dev, W_dev, seeds, v0, v1, **kw):
        K = kw.get("K") or wl.K
        prm, keep = self.params(wl, seeds, **kw)
        guard = Guarded()
        out = guard.make("logits", (wl.B * wl.T * K, v1 - v0), torch.float32, float("nan"))
        dmb.dm_debug_logits(self.ctx, prm, h_dev, W_dev, v0, v1, out)
        torch.cuda.synchronize()
        guard.check()
        return out.cpu().numpy()


def compare_path_ids(gpu_ids, ref, tol=1e-3, label=None):
    """Path tokens against the oracle's (`ref` = what oracle.verify / verify_js returned).  A token
    may differ from the oracle's only at a row whose oracle top-2 gap is below tol, and then it must
    be one of the tokens whose oracle value lies within tol of the row's maximum (the oracle lists
    them in ref["near"]): nothing else is a correct result.  Prints and returns
    (#rows that differ, #rows with gap < tol)."""
    gpu_ids = np.asarray(gpu_ids)
    ref_ids, gap, near = ref["path_ids"], ref["gap"], ref["near"]
    assert ref["near_tol"] >= tol, "ask the oracle for near_tol >= the tolerance of the comparison"
    assert gpu_ids.shape == ref_ids.shape
    mism = gpu_ids != ref_ids
    for idx in np.argwhere(mism):
        idx = tuple(int(x) for x in idx)
        assert gap[idx] < tol, f"path token differs at row {idx} with a clear top-1 (gap {gap[idx]:.3e}): " \
                               f"{int(gpu_ids[idx])} vs {int(ref_ids[idx])}"
        ids, deficit = near[idx]
        ok = ids[deficit <= tol]
        assert int(gpu_ids[idx]) in ok, f"row {idx}: token {int(gpu_ids[idx])} is not within {tol} of the " \
                                        f"oracle's maximum (candidates {ok.tolist()})"
    nflip, nnear = int(mism.sum()), int((gap < tol).sum())
    if label is not None:
        print(f"[{label}] rows={gap.size} near-tie rows(gap<{tol:g})={nnear} path-token flips={nflip}", flush=True)
    return nflip, nnear


# Tolerance of the JS values (float32 path against the float64 oracle).  The logits carry an
# absolute error of about 1e-5 (fp32 accumulation over d terms), so every ln p is off by up to
# that much; JS is second order in the log-ratio delta between a distribution and the centroid,
# dJS ~ (1/4) E|delta * err|, and the errors of the K paths and of their mean are independent
# and of both signs, so they average out over the vocabulary: expected |dJS| ~ 1e-5 * |delta| /
# (4 sqrt(V)) plus a relative error of a few 1e-7 per fp32 exp/log/sum.  Bound used: 2e-6 +
# 2e-4 * JS (observed on the MI355X: <= 2e-7 at every shape tested).
JS_ATOL, JS_RTOL = 2e-6, 2e-4


def compare_js(res, ref, draft, rule_js_only, path_flips, label=""):
    """JS values within tolerance; per-row decisions equal to the oracle's except where the
    oracle's Eq. (6) margin is inside the tolerance band (counted, printed).  Returns the
    number of such near-tie rows."""
    jh_ref, jd_ref = ref["js_heads"], ref["js_draft"]
    assert np.all(np.abs(res["js_heads"] - jh_ref) <= JS_ATOL + JS_RTOL * np.abs(jh_ref)), \
        f"{label}: js_heads off by up to {np.abs(res['js_heads'] - jh_ref).max():.3e}"
    has = draft >= 0
    assert np.all(res["js_draft"][~has] == -1.0)
    assert np.all(np.abs(res["js_draft"][has] - jd_ref[has]) <= JS_ATOL + JS_RTOL * np.abs(jd_ref[has])), \
        f"{label}: js_draft off by up to {np.abs(res['js_draft'][has] - jd_ref[has]).max():.3e}"
    band = 2 * (JS_ATOL + JS_RTOL * np.abs(np.where(has, jd_ref, 0.0)))
    near = has & (np.abs(ref["js_margin"]) <= band)
    # decisions: the GPU's own Eq. (6) outcome from its own values, then the rule
    gpu_js = has & (res["js_draft"] <= res["js_heads"].max(axis=-1))
    ref_js = has & (ref["js_margin"] >= 0)
    assert np.array_equal(gpu_js[~near], ref_js[~near]), f"{label}: Eq. (6) decision differs away from a tie"
    print(f"[{label}] rows={has.size} with draft={int(has.sum())} js-accept={int(ref_js.sum())} "
          f"near-tie rows={int(near.sum())} max|d js_heads|={np.abs(res['js_heads'] - jh_ref).max():.2e} "
          f"max|d js_draft|={np.abs(res['js_draft'][has] - jd_ref[has]).max() if has.any() else 0:.2e}", flush=True)
    return int(near.sum()), gpu_js


def check_graph_replays(enqueue, out, eager, between, reps=4):
    """Capture enqueue(stream) (one library call writing the tensors in `out`) in a HIP graph and
    replay it: every replay must reproduce `eager` (host arrays by the same keys), with eager work
    (`between()`) and synchronisations between the replays."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream
        enqueue(side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(torch.cuda.current_stream())
    for rep in range(reps):
        for v in out.values():
            v.fill_(7 if v.dtype == torch.uint8 else -1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in out.items():
            got, want = v.cpu().numpy(), eager[k]
            same = np.array_equal(got, want) if got.dtype.kind != "f" else np.array_equal(got, want, equal_nan=True)
            assert same, f"replay {rep}: {k}"
        between()
    del graph
