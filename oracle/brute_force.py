"""Brute-force checkers that pin the oracle (test infrastructure only, CPU only).

Written separately from evict_oracle.py, in a different formulation, so that a mistake in
one is not repeated in the other:

  * node_output_dense: a tree node is verified exactly as if its root path were a plain
    token sequence appended to the prefix (Sec. 2.1: the tree pass yields
    P(v | tokens before v) for every node). The path is run as an ordinary causal
    single-sequence decode, attention evaluated for the last position only, and the MoE
    evaluated densely: all experts computed, multiplied by a k-hot weight vector (Sec. 2.2).
  * accept_longest_matching_path: enumerate every root-to-node path and keep the longest
    one whose every edge carries the target's token (greedy case of Sec. 2.1).
  * best_prefix_exhaustive: enumerate all ancestor-closed node subsets; for every size k the
    best achievable sum of scores (Sec. 3.2.1 optimality claim) and the k maximising
    best_sum(k) / C(k) (Eq. 10).
"""
from __future__ import annotations

import itertools

import numpy as np


def _unit_rms(v, gain, eps):
    v = np.asarray(v, np.float64)
    out = np.empty_like(v)
    for r in range(v.shape[0]):
        out[r] = v[r] * gain / np.sqrt(np.dot(v[r], v[r]) / v.shape[1] + eps)
    return out


def _rotate_complex(vec, position, theta):
    """Rotary embedding in complex form: (v[i] + 1j*v[i+D/2]) * exp(1j*position*theta^(-2i/D))."""
    if not theta:
        return np.asarray(vec, np.float64)
    vec = np.asarray(vec, np.float64)
    D = vec.shape[-1]
    half = D // 2
    z = vec[..., :half] + 1j * vec[..., half:]
    freq = np.array([theta ** (-(2.0 * i) / D) for i in range(half)])
    z = z * np.exp(1j * position * freq)
    return np.concatenate([z.real, z.imag], axis=-1)


def node_output_dense(cfg, W, x_path, K, V, L):
    """x_path: [m, d] hidden rows of the root..node path (root first). K, V: [Hkv, >=L, D].
    Returns (out [d], h [d], top-k expert set, dense weight vector [E]) for the last row."""
    f = np.float64
    m = x_path.shape[0]
    gq = cfg.Hq // cfg.Hkv
    xn = _unit_rms(x_path, np.asarray(W["g_attn"], f), cfg.eps)
    # keys / values of the whole plain sequence: prefix cache, then the path tokens
    k_seq = [np.asarray(K, f)[:, :L]]
    v_seq = [np.asarray(V, f)[:, :L]]
    for s in range(m):
        kk = (np.asarray(W["wk"], f) @ xn[s]).reshape(cfg.Hkv, cfg.D)
        vv = (np.asarray(W["wv"], f) @ xn[s]).reshape(cfg.Hkv, cfg.D)
        k_seq.append(_rotate_complex(kk, L + s, cfg.theta)[:, None, :])
        v_seq.append(vv[:, None, :])
    k_seq = np.concatenate(k_seq, axis=1)      # [Hkv, L+m, D]
    v_seq = np.concatenate(v_seq, axis=1)
    qq = (np.asarray(W["wq"], f) @ xn[-1]).reshape(cfg.Hq, cfg.D)
    qq = _rotate_complex(qq, L + m - 1, cfg.theta)
    heads = []
    for hh in range(cfg.Hq):
        g = hh // gq
        logit = np.array([np.dot(k_seq[g, t], qq[hh]) for t in range(L + m)]) / np.sqrt(cfg.D)
        e = np.exp(logit - np.max(logit))
        prob = e / np.sum(e)
        heads.append(sum(prob[t] * v_seq[g, t] for t in range(L + m)))
    o = np.concatenate(heads)
    h = np.asarray(x_path[-1], f) + np.asarray(W["wo"], f) @ o
    hn = _unit_rms(h[None, :], np.asarray(W["g_moe"], f), cfg.eps)[0]
    scores = np.asarray(W["wg"], f) @ hn
    top = np.argsort(-scores, kind="stable")[:cfg.k]
    dense_w = np.zeros(cfg.E, f)
    ex = np.exp(scores[top] - scores[top].max())
    dense_w[top] = ex / ex.sum()
    all_out = np.zeros((cfg.E, cfg.d), f)
    for e_ in range(cfg.E):
        gte = np.asarray(W["w_gate"][e_], f) @ hn
        upp = np.asarray(W["w_up"][e_], f) @ hn
        all_out[e_] = np.asarray(W["w_down"][e_], f) @ (gte / (1.0 + np.exp(-gte)) * upp)
    out = h + dense_w @ all_out
    for s_ in range(getattr(cfg, "n_shared", 0)):
        gte = np.asarray(W["ws_gate"][s_], f) @ hn
        upp = np.asarray(W["ws_up"][s_], f) @ hn
        out = out + np.asarray(W["ws_down"][s_], f) @ (gte / (1.0 + np.exp(-gte)) * upp)
    return out, h, set(int(t) for t in top), dense_w


def root_path(parent, i):
    path = []
    while i >= 0:
        path.append(i)
        i = int(parent[i])
    return path[::-1]


def accept_longest_matching_path(parent, draft_tok, target_next):
    """Among all root paths whose every edge (u -> c) has draft_tok[c] == target_next[u], the
    longest (unique when sibling tokens are distinct). Returns the list of node ids."""
    n = len(parent)
    best = [0]
    for v in range(n):
        p = root_path(parent, v)
        ok = all(draft_tok[p[j + 1]] == target_next[p[j]] for j in range(len(p) - 1))
        if ok and len(p) > len(best):
            best = p
    return best


def best_prefix_exhaustive(parent, score, cost, kmax):
    """Enumerate every ancestor-closed subset containing the root. Returns
    (best_sum[k] for k=1..min(n,kmax) as float64, argmax_k best_sum[k]/cost[k] (smallest k))."""
    n = len(parent)
    kk = min(n, kmax)
    best = np.full(kk + 1, -np.inf)
    others = list(range(1, n))
    for r in range(0, kk):
        for sub in itertools.combinations(others, r):
            s = set(sub) | {0}
            if all(parent[v] in s for v in sub):
                tot = float(sum(np.float64(score[v]) for v in s))
                if tot > best[r + 1]:
                    best[r + 1] = tot
    util = [best[k] / float(cost[k]) for k in range(1, kk + 1)]
    kbest = int(np.argmax(util)) + 1
    return best[1:], kbest, util
