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


class Runner:
    """Owns a context sized for one workload shape."""

    def __init__(self, max_rows, max_d, max_V):
        self.ctx = dmb.dm_create(0, max_rows, max_d, max_V)

    def close(self):
        if self.ctx is not None:
            dmb.dm_destroy(self.ctx)
            self.ctx = None

    def params(self, wl, seeds, p=None, step=0, rule=dmb.DM_RULE_ANY, flags=0, parent=None, K=None):
        dtype = dmb.DM_BF16 if wl.dtype == "bf16" else dmb.DM_F32
        return dmb.make_params(wl.B, wl.T, wl.K if K is None else K, wl.d, wl.V, dtype,
                               wl.p if p is None else p, [int(s) for s in seeds], step=step, rule=rule,
                               flags=flags, parent=parent)

    def verify(self, wl, h_dev, W_dev, draft, seeds, parent=None, **kw):
        K = kw.get("K") or wl.K
        B, T = wl.B, wl.T
        dev = "cuda"
        par_dev = None if parent is None else torch.from_numpy(np.ascontiguousarray(parent, dtype=np.int32)).cuda()
        prm, keep = self.params(wl, seeds, parent=par_dev, **kw)
        draft_dev = torch.from_numpy(np.ascontiguousarray(draft, dtype=np.int32)).cuda()
        out = dict(
            accept_len=torch.full((B,), -7, dtype=torch.int32, device=dev),
            best_node=torch.full((B,), -7, dtype=torch.int32, device=dev),
            accept_mask=torch.full((B, T), 9, dtype=torch.uint8, device=dev),
            hit=torch.full((B, T), 9, dtype=torch.uint8, device=dev),
            path_ids=torch.full((B, T, K), -7, dtype=torch.int32, device=dev),
            vote_ids=torch.full((B, T), -7, dtype=torch.int32, device=dev),
            vote_cnt=torch.full((B, T), -7, dtype=torch.int32, device=dev),
        )
        dmb.dropmatch_verify(self.ctx, prm, h_dev, W_dev, draft_dev, **out)
        torch.cuda.synchronize()
        del keep
        return {k: v.cpu().numpy() for k, v in out.items()}

    def masks(self, wl, seeds, **kw):
        K = kw.get("K") or wl.K
        nw = (wl.d + 31) // 32
        prm, keep = self.params(wl, seeds, **kw)
        bits = torch.full((wl.B, wl.T, K, nw), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        dmb.dm_debug_masks(self.ctx, prm, bits)
        torch.cuda.synchronize()
        return bits.cpu().numpy().view(np.uint32)

    def logits(self, wl, h_dev, W_dev, seeds, v0, v1, **kw):
        K = kw.get("K") or wl.K
        prm, keep = self.params(wl, seeds, **kw)
        out = torch.full((wl.B * wl.T * K, v1 - v0), float("nan"), dtype=torch.float32, device="cuda")
        dmb.dm_debug_logits(self.ctx, prm, h_dev, W_dev, v0, v1, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()


def compare_path_ids(gpu_ids, ref_ids, gap, tol=1e-3):
    """Path tokens must be equal except where the oracle's top-2 logit gap is below tol.
    Returns (#rows that differ, #rows with gap < tol)."""
    mism = gpu_ids != ref_ids
    bad = mism & (gap >= tol)
    assert not bad.any(), f"{int(bad.sum())} path tokens differ at rows with a clear top-1 " \
                          f"(first: {np.argwhere(bad)[0].tolist()})"
    return int(mism.sum()), int((gap < tol).sum())
