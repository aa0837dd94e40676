"""CPU checks of the comparison helpers the GPU parity tests rely on: a mistake planted in a copy
of the oracle's own result must be caught, a legitimate near-tie flip must pass."""
import numpy as np
import pytest

from oracle import dropmatch_oracle as orc
from paper_2603_03333_amd import workloads as wk

pytest.importorskip("torch")
import torch  # noqa: E402
from gpu_harness import GUARD, Guarded, compare_path_ids  # noqa: E402


def _near_tie_problem():
    """Two vocabulary rows made equal up to 2e-4 in the row that wins position 0, so that the oracle
    reports a near tie there with exactly two candidates."""
    wl = wk.Workload("tie", d=32, V=50, dtype="f32", B=1, T=2, K=3, p=0.0, data_seed=5)
    W, h = wk.make_weight(wl, sigma=0.1).astype(np.float64), wk.make_hidden(wl).astype(np.float64)
    top = int(np.argmax(W @ h[0, 0]))
    other = (top + 7) % wl.V
    W[other] = W[top]
    W[other, 0] -= 2e-4 / h[0, 0, 0] if h[0, 0, 0] > 0 else -2e-4 / -h[0, 0, 0]
    seeds = np.array([1], dtype=np.uint64)
    ref = orc.verify(h, W, np.zeros((1, 2), int), seeds, wl.K, 0.0)
    return ref, top, other


def test_tokens_within_hand_case():
    ids, deficit = orc.tokens_within(np.array([1.0, 3.0, 2.9995, 0.0, 3.0]), 1e-3)
    assert ids.tolist() == [1, 2, 4] and np.allclose(deficit, [0.0, 5e-4, 0.0])
    ids, _ = orc.tokens_within(np.array([1.0, 3.0, 2.9995, 0.0, 3.0]), 1e-4)
    assert ids.tolist() == [1, 4]


def test_compare_path_ids_accepts_only_the_near_tie_candidates():
    ref, top, other = _near_tie_problem()
    assert (ref["gap"][0, 0] < 1e-3).all() and (ref["gap"][0, 1] > 1e-3).all()
    ids = {int(x) for x in ref["near"][(0, 0, 0)][0]}
    assert ids == {top, other}
    good = ref["path_ids"].copy()
    assert compare_path_ids(good, ref) == (0, 3)
    runner_up = other if ref["path_ids"][0, 0, 0] == top else top
    good[0, 0, 1] = runner_up                               # the other candidate of a near tie: valid
    assert compare_path_ids(good, ref) == (1, 3)
    bad = ref["path_ids"].copy()
    bad[0, 0, 1] = (top + 1) % 50 if (top + 1) % 50 != other else (top + 2) % 50
    with pytest.raises(AssertionError, match="not within"):  # garbage at a near-tie row
        compare_path_ids(bad, ref)
    bad = ref["path_ids"].copy()
    bad[0, 0, 2] = -1                                       # an unwritten sentinel at a near-tie row
    with pytest.raises(AssertionError, match="not within"):
        compare_path_ids(bad, ref)
    bad = ref["path_ids"].copy()
    bad[0, 1, 0] = runner_up                                # any change at a row with a clear top-1
    with pytest.raises(AssertionError, match="clear top-1"):
        compare_path_ids(bad, ref)
    with pytest.raises(AssertionError, match="near_tol"):    # the oracle must have listed candidates that far out
        compare_path_ids(good, ref, tol=0.5)


def test_sampled_values_agree_with_sampled_token():
    rng = np.random.default_rng(3)
    l = rng.normal(size=40)
    g = orc.gumbel_noise(rng.uniform(0.01, 0.99, size=40))
    for top_p in (None, 0.6):
        y = orc.sampled_values(l, 0.7, g, top_p)
        tok, gap = orc.sampled_token(l, 0.7, g, top_p)
        assert tok == int(np.argmax(y))
        assert orc.tokens_within(y, 0.0)[0].tolist() == [tok]
    inside = orc.nucleus(l / 0.7, 0.6)[0]
    assert np.isneginf(y[~inside]).all() and np.isfinite(y[inside]).all()


@pytest.mark.parametrize("dtype,fill", [(torch.int32, -7), (torch.uint8, 9), (torch.float32, float("nan"))])
def test_guarded_outputs_catch_a_write_one_element_outside(dtype, fill):
    g = Guarded(device="cpu")
    v = g.make("x", (3, 5), dtype, fill)
    assert v.shape == (3, 5) and v.is_contiguous()
    v.fill_(1)                                   # writing every own element is fine
    g.check()
    buf = g.bufs["x"][0]
    for where in (GUARD - 1, GUARD + 15):        # the element just before and just after
        old = buf[where].clone()
        buf[where] = 1
        with pytest.raises(AssertionError, match="outside the output buffer"):
            g.check()
        buf[where] = old
    g.check()
