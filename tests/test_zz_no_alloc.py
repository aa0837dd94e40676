"""The allocation-free entry point, dropmatch_verify_static (for callers that cannot allocate device
memory), against dropmatch_verify on a context: identical outputs, call after call, the second call
on a smaller input than the first (the fixed workspace keeps the first call's contents), through the
C ABI.  Also its limits."""
import numpy as np
import pytest

from paper_2603_03333_amd import workloads as wk

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2603_03333_amd import binding as dmb  # noqa: E402
from gpu_harness import Guarded, Runner, to_device  # noqa: E402

KEYS = ("accept_len", "best_node", "accept_mask", "hit", "path_ids", "vote_ids", "vote_cnt")


def _static_verify(wl, h_dev, W_dev, draft, seeds, parent=None, **kw):
    B, T, K = wl.B, wl.T, wl.K
    dtype = dmb.DM_BF16 if wl.dtype == "bf16" else dmb.DM_F32
    par_dev = None if parent is None else torch.from_numpy(np.ascontiguousarray(parent, dtype=np.int32)).cuda()
    prm, keep = dmb.make_params(B, T, K, wl.d, wl.V, dtype, wl.p, [int(s) for s in seeds], parent=par_dev, **kw)
    draft_dev = torch.from_numpy(np.ascontiguousarray(draft, dtype=np.int32)).cuda()
    guard = Guarded()
    out = dict(accept_len=guard.make("accept_len", (B,), torch.int32, -7),
               best_node=guard.make("best_node", (B,), torch.int32, -7),
               accept_mask=guard.make("accept_mask", (B, T), torch.uint8, 9),
               hit=guard.make("hit", (B, T), torch.uint8, 9),
               path_ids=guard.make("path_ids", (B, T, K), torch.int32, -7),
               vote_ids=guard.make("vote_ids", (B, T), torch.int32, -7),
               vote_cnt=guard.make("vote_cnt", (B, T), torch.int32, -7))
    dmb.dropmatch_verify_static(0, prm, h_dev, W_dev, draft_dev, **out)
    torch.cuda.synchronize()
    guard.check()
    del keep
    return {k: v.cpu().numpy() for k, v in out.items()}


def _pair(wl, seed0, parent=None, **kw):
    """The same problem through both entry points."""
    W, h = wk.make_weight(wl, sigma=0.1), wk.make_hidden(wl)
    seeds = wk.make_seeds(wl, base_seed=seed0)
    draft = np.random.default_rng(seed0).integers(0, wl.V, size=(wl.B, wl.T)).astype(np.int32)
    hd, Wd = to_device(h, wl.dtype), to_device(W, wl.dtype)
    got = _static_verify(wl, hd, Wd, draft, seeds, parent=parent, **kw)
    r = Runner(wl.rows, wl.d, wl.V)
    try:
        want = r.verify(wl, hd, Wd, draft, seeds, parent=parent, **kw)
    finally:
        r.close()
    for k in KEYS:
        assert np.array_equal(got[k], want[k]), f"{wl.name}: {k} differs between the two entry points"
    assert (got["path_ids"] >= 0).all() and (got["path_ids"] < wl.V).all()
    return got


@pytest.mark.parametrize("first,second", [
    # (d, V, dtype, B, T, K) of the first call, then of a smaller second call
    ((512, 3000, "bf16", 2, 8, 8), (256, 1000, "bf16", 1, 5, 5)),        # W-streaming kernel, fused acceptance step
    ((256, 2500, "bf16", 4, 8, 20), (128, 777, "bf16", 1, 3, 16)),       # 256 x 256 tiles (640 rows), then 48 rows
    ((100, 130, "f32", 2, 4, 6), (37, 65, "f32", 1, 2, 3)),              # generic kernel
])
def test_static_entry_equals_context_entry_two_calls_in_a_row(first, second):
    for n, (d, V, dtype, B, T, K) in enumerate((first, second)):
        wl = wk.Workload(f"static{n}", d=d, V=V, dtype=dtype, B=B, T=T, K=K, p=0.1, bonus=True, data_seed=400 + n)
        for rule in (dmb.DM_RULE_ANY, dmb.DM_RULE_MAJORITY):
            _pair(wl, seed0=31 + n, rule=rule)


def test_static_entry_head8b_shape_then_smaller():
    """The benchmark's shape (128 rows, d = 4096, V = 128256: 1 MB of masked rows) and then 40 rows."""
    big = wk.CONFIGS["head8b"]
    _pair(big, seed0=5)
    _pair(big.with_(K=5), seed0=6)
    # sampled path tokens and the clean last path use the seeds and flags of the fixed workspace too
    small = wk.Workload("static-s", d=256, V=3000, dtype="bf16", B=2, T=6, K=8, p=0.2, bonus=True, data_seed=77)
    _pair(small, seed0=7, flags=dmb.DM_FLAG_SAMPLE_PATHS | dmb.DM_FLAG_CLEAN_LAST_PATH, temperature=0.8)


def test_static_entry_tree_mode():
    wl = wk.Workload("static-tree", d=256, V=2000, dtype="bf16", B=3, T=12, K=8, p=0.1, tree=True, data_seed=9)
    parent = wk.make_tree_parents(wl, max_depth=4, max_branch=3)
    _pair(wl, seed0=11, parent=parent)


def test_static_entry_limits():
    wl = wk.Workload("lim", d=4096, V=512, dtype="bf16", B=1, T=8, K=16, p=0.1)
    h = torch.zeros((1, 8, 4096), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((512, 4096), dtype=torch.bfloat16, device="cuda")
    draft = torch.zeros((64, 64), dtype=torch.int32, device="cuda")
    out = torch.zeros(4096, dtype=torch.int32, device="cuda")

    def call(**over):
        a = dict(B=1, T=8, K=16, d=4096, V=512, dtype=dmb.DM_BF16, p=0.1, seeds=[1], rule=dmb.DM_RULE_ANY, flags=0)
        a.update(over)
        seeds = a.pop("seeds") * a["B"]
        prm, keep = dmb.make_params(a.pop("B"), a.pop("T"), a.pop("K"), a.pop("d"), a.pop("V"), a.pop("dtype"),
                                    a.pop("p"), seeds, **a)
        dmb.dropmatch_verify_static(0, prm, h, W, draft, out)

    call()                                                   # inside every limit
    with pytest.raises(dmb.DropMatchError) as e:             # 2049 rows
        call(B=1, T=1, K=1024, d=64)                         # fine: 1024 rows ...
        call(B=3, T=1, K=683, d=64)                          # ... 2049 are not
    assert e.value.status == dmb.DM_EINVAL and "DM_STATIC_MAX_ROWS" in e.value.message
    with pytest.raises(dmb.DropMatchError) as e:             # 2048 rows x 4096 x 2 bytes = 16 MB of masked rows
        call(B=2, T=8, K=128)
    assert e.value.status == dmb.DM_EINVAL and "DM_STATIC_MAX_WS_BYTES" in e.value.message
    with pytest.raises(dmb.DropMatchError) as e:
        call(rule=dmb.DM_RULE_JS_OR_MAJORITY)
    assert e.value.status == dmb.DM_EUNSUPPORTED
    with pytest.raises(dmb.DropMatchError) as e:
        call(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=1.0, top_p=0.9)
    assert e.value.status == dmb.DM_EUNSUPPORTED
    with pytest.raises(dmb.DropMatchError) as e:
        call(p=1.5)
    assert e.value.status == dmb.DM_EINVAL
    torch.cuda.synchronize()
    call()                                                   # still usable after the rejected calls
    torch.cuda.synchronize()
