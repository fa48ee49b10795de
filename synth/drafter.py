"""Synthetic stand-in for the draft model in a multi-iteration speculative loop (inputs only).

Each iteration gets a draft tree with per-node draft probabilities, correlated hidden states,
draft token ids, and the target's next-token id at every node. The target ids are drawn so that
the drafter is calibrated in the sense Eq. 7-8 assume: at node u the target continues with child
c with probability q(c) (children's q are scaled down together when they sum to more than 1) and
with none of the children otherwise, so a root path is accepted with the product of its q's.
Nothing here evaluates the method; the draws are inputs to both the GPU loop and the oracle.
"""
from __future__ import annotations

import numpy as np

from .inputs import ModelCfg, hidden_states, philox, tree_bfs_random, tree_eagle_style, draft_probs


def tree_topk_drafter(n: int, g: np.random.Generator, first_branch: int = 4, branch: int = 2, max_depth: int = 6,
                      support: int = 32, sharpness: float = 2.0):
    """Draft tree whose sibling probabilities are parts of one distribution, as a real drafter's
    are: at an expanded node a categorical over `support` candidates is drawn (softmax of
    sharpness * N(0,1)) and its most likely entries become the children, so siblings sum to at
    most 1. Expansion order as in tree_eagle_style: the root gets `first_branch` children, then
    the childless node of depth < max_depth with the highest cumulative probability (ties:
    lowest index) gets `branch`, until n nodes exist. Returns (parent, q)."""
    parent, q, cum, dep, has_child = [-1], [1.0], [1.0], [0], [False]

    def expand(v: int, m: int):
        has_child[v] = True
        z = sharpness * g.standard_normal(support)
        p = np.exp(z - z.max())
        p = np.sort(p / p.sum())[::-1]
        for j in range(m):
            if len(parent) >= n:
                return
            parent.append(v)
            q.append(float(p[j]))
            cum.append(cum[v] * float(p[j]))
            dep.append(dep[v] + 1)
            has_child.append(False)

    if n > 1:
        expand(0, first_branch)
    while len(parent) < n:
        cand = [i for i in range(len(parent)) if not has_child[i] and dep[i] < max_depth]
        if not cand:
            break
        expand(max(cand, key=lambda i: (cum[i], -i)), branch)
    while len(parent) < n:  # every leaf at max depth: hang the rest under the root with small mass
        parent.append(0)
        q.append(1e-3)
    return np.asarray(parent, dtype=np.int32), np.asarray(q, dtype=np.float32)


def draft_iteration(cfg: ModelCfg, n: int, seed: int, it: int, sigma: float, vocab: int, tree: str = "topk") -> dict:
    g = philox(seed, 5000 + it)
    if tree == "topk":
        parent, q = tree_topk_drafter(n, g)
    elif tree == "eagle":
        parent, q = tree_eagle_style(n, g)
    else:
        parent = tree_bfs_random(n, g)
        q = draft_probs(n, g, "beta22")
    q = np.asarray(q, np.float32)
    x = hidden_states(parent, cfg.d, sigma, g, cfg.dtype)
    children = [[] for _ in range(n)]
    for i in range(1, n):
        children[parent[i]].append(i)
    tok = np.zeros(n, np.int32)
    target_next = np.zeros(n, np.int32)
    tok[0] = int(g.integers(0, vocab))
    for u in range(n):
        ch = children[u]
        ids = g.choice(vocab - 1, size=len(ch), replace=False).astype(np.int32) if ch else np.zeros(0, np.int32)
        for c, t in zip(ch, ids):
            tok[c] = t                      # distinct ids in [0, vocab - 1); vocab - 1 is carried by no child
        pc = np.asarray([q[c] for c in ch], np.float64)
        pc = pc / max(1.0, pc.sum())
        r = g.random()
        target_next[u] = vocab - 1
        acc = 0.0
        for c, p in zip(ch, pc):
            acc += p
            if r < acc:
                target_next[u] = tok[c]
                break
    return {"parent": parent.astype(np.int32), "q": q, "x": x, "tok": tok, "target_next": target_next}
