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


def draft_iteration(cfg: ModelCfg, n: int, seed: int, it: int, sigma: float, vocab: int, tree: str = "eagle") -> dict:
    g = philox(seed, 5000 + it)
    if tree == "eagle":
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
