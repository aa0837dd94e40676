"""Seeded synthetic inputs for the DropMatch verify step.

This module builds INPUTS only (weights, hidden states, draft tokens, draft trees);
it contains none of the method's arithmetic - no mask, no LM-head product, no
acceptance rule - so that the CPU oracle and the HIP path can both be fed from it
without sharing anything that is under test.  Where a recipe needs the greedy
(no-dropout) token of a row in order to plant matching draft tokens, the caller
passes those tokens in.

Shapes follow the model families the paper evaluates (Llama-3.1 8B/70B and Qwen3
heads: d in {4096, 8192}, V in {128256, 151936}), draft lengths 5-10 plus a bonus
row, and tree decoding as used with EAGLE-3 (Experiments, "Speculative Decoding
with DropMatch" and the EAGLE-3 subsection).  Values are i.i.d. Gaussian stand-ins:
the paper's datasets and checkpoints are not available.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    d: int
    V: int
    dtype: str            # "f32" or "bf16": storage type of h and W
    B: int
    T: int                # rows of h per sequence (chain positions incl. bonus, or tree nodes)
    K: int
    p: float
    bonus: bool = False   # chain: last row carries no draft token (draft id -1)
    tree: bool = False    # rows are nodes of a draft tree with parent indices
    data_seed: int = 1000

    @property
    def rows(self) -> int:
        return self.B * self.T * self.K

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five benchmark configurations.
CONFIGS = {
    "tiny": Workload("tiny", d=256, V=4096, dtype="f32", B=1, T=5, K=8, p=0.1, data_seed=1000),
    "head8b": Workload("head8b", d=4096, V=128256, dtype="bf16", B=1, T=8, K=16, p=0.1,
                       bonus=True, data_seed=1001),
    "bigvocab": Workload("bigvocab", d=4096, V=151936, dtype="bf16", B=4, T=8, K=32, p=0.1,
                         bonus=True, data_seed=1002),
    "tree": Workload("tree", d=4096, V=128256, dtype="bf16", B=8, T=64, K=16, p=0.1,
                     tree=True, data_seed=1003),
    "batched": Workload("batched", d=8192, V=128256, dtype="bf16", B=32, T=8, K=16, p=0.1,
                        bonus=True, data_seed=1004),
}


# --------------------------------------------------------------------------- #
# bfloat16 storage (round-to-nearest-even on the upper 16 bits of a float32)
# --------------------------------------------------------------------------- #
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bfloat16 bit patterns, round to nearest even.
    Inputs must be finite (the generators here only produce finite values)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in bfloat16."""
    return bf16_to_f32(bf16_bits(x))


def _round_to_bf16_inplace(x: np.ndarray) -> None:
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u += np.uint32(0x7FFF)
    u += lsb
    u &= np.uint32(0xFFFF0000)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- #
# W, h
# --------------------------------------------------------------------------- #
def make_weight(wl: Workload, sigma: float = 0.02) -> np.ndarray:
    """W[V, d] ~ N(0, sigma) as float32 holding values of the storage dtype."""
    if wl.dtype not in ("bf16", "f32"):
        raise ValueError(wl.dtype)
    rng = np.random.Generator(np.random.PCG64(wl.data_seed))
    W = np.empty((wl.V, wl.d), dtype=np.float32)
    step = 8192                      # row blocks: one sequential stream, no large temporaries
    for r0 in range(0, wl.V, step):
        blk = W[r0:r0 + step]
        rng.standard_normal(out=blk, dtype=np.float32)
        blk *= np.float32(sigma)
        if wl.dtype == "bf16":
            _round_to_bf16_inplace(blk)
    return W


def make_hidden(wl: Workload) -> np.ndarray:
    """h[B, T, d] ~ N(0, 1) as float32 holding values of the storage dtype."""
    rng = np.random.Generator(np.random.PCG64(wl.data_seed + 7919))
    return _store(rng.standard_normal((wl.B, wl.T, wl.d), dtype=np.float32), wl.dtype)


def make_planted_hidden(wl: Workload, W: np.ndarray, alpha: float):
    """Hidden states with a known dominant token: h_t = alpha * W[y_t] / |W[y_t]| + eps,
    eps ~ N(0, 1).  Models the peaked next-token distributions of a real LM (the
    paper's agreement table: all K = 5 paths agree at 98.4 % of positions).
    Returns (h[B,T,d], planted token ids[B,T])."""
    rng = np.random.Generator(np.random.PCG64(wl.data_seed + 104729))
    y = rng.integers(0, wl.V, size=(wl.B, wl.T))
    rows = W[y].astype(np.float64)
    rows /= np.linalg.norm(rows, axis=-1, keepdims=True)
    eps = rng.standard_normal((wl.B, wl.T, wl.d))
    return _store((alpha * rows + eps).astype(np.float32), wl.dtype), y.astype(np.int32)


def make_seeds(wl: Workload, base_seed: int = 0) -> np.ndarray:
    """Independent mask seed per sequence: base_seed + b."""
    return (np.uint64(base_seed) + np.arange(wl.B, dtype=np.uint64)).astype(np.uint64)


# --------------------------------------------------------------------------- #
# draft tokens (chain)
# --------------------------------------------------------------------------- #
def make_draft_ids(wl: Workload, greedy: Optional[np.ndarray]) -> np.ndarray:
    """draft_ids[B, T]: uniform in [0, V); then each row, independently with
    probability 1/2, is replaced by the caller-supplied greedy token of that row
    (so about half of the draft tokens agree with the undropped head).  With a
    bonus row the last entry is -1 (nothing to verify there)."""
    rng = np.random.Generator(np.random.PCG64(wl.data_seed + 15485863))
    ids = rng.integers(0, wl.V, size=(wl.B, wl.T)).astype(np.int32)
    forced = rng.random((wl.B, wl.T)) < 0.5
    if greedy is not None:
        ids = np.where(forced, np.asarray(greedy, dtype=np.int32), ids)
    if wl.bonus:
        ids[:, -1] = -1
    return np.ascontiguousarray(ids, dtype=np.int32)


# --------------------------------------------------------------------------- #
# draft distributions (inputs of the distribution-level rule)
# --------------------------------------------------------------------------- #
DRAFT_NOISE_LEVELS = (0.1, 0.3, 0.42, 0.6)


def make_draft_probs(wl: Workload, clean_logits: np.ndarray, topk: int = 0) -> np.ndarray:
    """draft_probs[B, T, V] float32: a stand-in for the draft model's next-token
    distribution at every row.  The caller supplies the undropped head logits of the
    row (clean_logits[B, T, V]); the draft is that plus i.i.d. Gaussian noise whose
    standard deviation is drawn per row from DRAFT_NOISE_LEVELS (close drafts and far
    drafts in one batch), normalised to a distribution.  With topk > 0 everything but
    the topk largest entries is set to exactly 0 and the rest renormalised (drafts that
    sample from a truncated distribution)."""
    rng = np.random.Generator(np.random.PCG64(wl.data_seed + 86028121))
    B, T, V = clean_logits.shape
    out = np.empty((B, T, V), dtype=np.float32)
    levels = rng.integers(0, len(DRAFT_NOISE_LEVELS), size=(B, T))
    for b in range(B):
        for t in range(T):
            z = clean_logits[b, t].astype(np.float64)
            z = z + DRAFT_NOISE_LEVELS[int(levels[b, t])] * rng.standard_normal(V)
            e = np.exp(z - z.max())
            if 0 < topk < V:
                cut = np.partition(e, V - topk)[V - topk]
                e[e < cut] = 0.0
            out[b, t] = (e / e.sum()).astype(np.float32)
    return out


# --------------------------------------------------------------------------- #
# draft trees
# --------------------------------------------------------------------------- #
def make_tree_parents(wl: Workload, max_depth: int = 6, max_branch: int = 4) -> np.ndarray:
    """parent[B, T] for draft trees of exactly T nodes in topological (BFS) order:
    node 0 is the root (parent -1); depth <= max_depth; at most max_branch children
    per node; a spine root -> depth max_depth is laid first so the full depth is
    always reachable, the remaining nodes attach to random eligible nodes."""
    rng = np.random.Generator(np.random.PCG64(wl.data_seed + 32452843))
    T = wl.T
    out = np.full((wl.B, T), -1, dtype=np.int32)
    for b in range(wl.B):
        par = [-1]
        depth = [0]
        nchild = [0]
        spine = min(max_depth, T - 1)
        for k in range(spine):                      # nodes 1..spine form a path
            par.append(k); depth.append(k + 1); nchild.append(0); nchild[k] += 1
        while len(par) < T:
            elig = [n for n in range(len(par)) if depth[n] < max_depth and nchild[n] < max_branch]
            q = int(elig[rng.integers(0, len(elig))])
            par.append(q); depth.append(depth[q] + 1); nchild.append(0); nchild[q] += 1
        # renumber into BFS order (stable by depth) so that parent[n] < n holds
        order = sorted(range(T), key=lambda n: (depth[n], n))
        new_of = {old: new for new, old in enumerate(order)}
        for old in range(T):
            out[b, new_of[old]] = -1 if par[old] < 0 else new_of[par[old]]
    return out


def make_tree_draft_ids(wl: Workload, parent: np.ndarray, greedy: Optional[np.ndarray]) -> np.ndarray:
    """Token of every tree node: uniform in [0, V), children of one parent distinct (while V allows);
    then, for every parent independently with probability 1/2, its first child gets
    the caller-supplied greedy token of the PARENT row (row n predicts n's children).
    The root's token is -1 (it is the last committed token, never verified)."""
    rng = np.random.Generator(np.random.PCG64(wl.data_seed + 49979687))
    B, T = parent.shape
    ids = np.zeros((B, T), dtype=np.int32)
    for b in range(B):
        ids[b, 0] = -1
        first_child = {}
        used = {}
        for n in range(1, T):
            q = int(parent[b, n])
            first_child.setdefault(q, n)
            tok = int(rng.integers(0, wl.V))
            # distinct among siblings as long as the vocabulary has unused tokens left for them
            while tok in used.setdefault(q, set()) and len(used[q]) < wl.V:
                tok = int(rng.integers(0, wl.V))
            used[q].add(tok)
            ids[b, n] = tok
        for q, n in sorted(first_child.items()):
            if rng.random() < 0.5 and greedy is not None:
                g = int(greedy[b, q])
                sibs = [m for m in range(1, T) if int(parent[b, m]) == q and m != n]
                if all(int(ids[b, m]) != g for m in sibs):
                    ids[b, n] = g
    return ids


def chain_as_tree(draft_chain: np.ndarray):
    """Re-express a chain whose last row is a bonus row as a degenerate tree over
    the same rows: node n has parent n-1 and carries the token that chain row n-1
    verifies.  Returns (parent[B,T], draft_tree[B,T])."""
    B, T = draft_chain.shape
    parent = np.tile(np.arange(-1, T - 1, dtype=np.int32), (B, 1))
    tree = np.full((B, T), -1, dtype=np.int32)
    tree[:, 1:] = draft_chain[:, :-1]
    return parent, tree
