"""CPU oracle for target-side verification of a draft token tree on a sparse MoE layer.

TEST INFRASTRUCTURE ONLY. Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg may import this module; the product path (the HIP library) never does and shares no code
with it.

It is the plain definition of what the verification step computes, evaluated slowly with
numpy in float64 on the (already storage-rounded) inputs:

  * tree verification in one pass, each node attending to the prefix and to its own
    ancestors (Sec. 2.1, Fig. 4(c));
  * router scores W_g h, TopK, normalisation of the selected scores by softmax, weighted sum
    of the selected experts (Sec. 2.2, Eq. 4);
  * the union of activated experts over all verified nodes (Eq. 5);
  * node scores as products of draft probabilities along the root path (Eq. 7), their sum
    as the estimated accepted length (Eq. 8), top-k pruning by cumulative score
    (Sec. 3.2.1), and k* = argmax_k Ehat[A(T_k)] / C(k) (Eq. 10) evaluated as
    cumulative sums, element-wise division and argmax (Sec. 3.2.3);
  * greedy (temperature 0) acceptance, the deterministic case of the sequential sibling
    rule of Sec. 2.1, and the rule itself under sampling (Eq. 3: accept a child with its
    current probability, on rejection remove its mass and renormalise, after the last
    sibling draw from the residual);
  * the exact expected accepted length (Eq. 6) and the expected number of distinct experts
    (App. A, Eq. 11) used as closed forms by the tests.

Transformer-layer facts the paper leaves to the architecture (RMSNorm, rotary positions at
context_length + depth, grouped-query attention, SiLU-gated expert MLP) are the textbook
definitions. No blocking, fusion or reordering: a reader can check each function by eye.

Pins (tests/test_oracle_pins.py, tests/test_select_accept_pins.py): brute-force per-node
dense evaluation of each root path, chain tree == causal decode, library attention / top-k /
matmul cross-checks, closed forms for chains, exhaustive enumeration of root-closed subsets,
Eq. 11 Monte-Carlo, the paper's Table 4 cost rows. No function here is parity-unpinned.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64
F32 = np.float32


# --------------------------------------------------------------------------------------
# storage rounding at tensor hand-offs (bf16 configurations only)
# --------------------------------------------------------------------------------------
def round_bf16(x):
    """Round to the nearest bf16 value (ties to even); result returned as float64."""
    u = np.ascontiguousarray(x, dtype=F32).view(np.uint32)
    u = (u + (((u >> 16) & 1) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return u.view(F32).astype(F64).reshape(np.shape(x))


def handoff(x, act):
    """Activations are stored in the model's storage type between stages: identity for
    "f32"/"f64" evaluation, bf16 rounding for "bf16"."""
    if act == "bf16":
        return round_bf16(x)
    if act == "f32":
        return np.asarray(x, dtype=F64).astype(F32).astype(F64)
    return np.asarray(x, dtype=F64)


# --------------------------------------------------------------------------------------
# tree structure (Sec. 2.1; mask of Fig. 4(c))
# --------------------------------------------------------------------------------------
def tree_ancestors(parent):
    """anc[i, j] is True iff j lies on the path root..i (i itself included); depth[i] is the
    number of edges from the root. Requires parent[0] == -1 and parent[i] < i."""
    n = len(parent)
    assert n >= 1 and parent[0] == -1
    anc = np.zeros((n, n), dtype=bool)
    depth = np.zeros(n, dtype=np.int64)
    anc[0, 0] = True
    for i in range(1, n):
        p = int(parent[i])
        assert 0 <= p < i
        anc[i] = anc[p]
        anc[i, i] = True
        depth[i] = depth[p] + 1
    return anc, depth


# --------------------------------------------------------------------------------------
# layer pieces
# --------------------------------------------------------------------------------------
def rmsnorm(x, gain, eps):
    x = np.asarray(x, dtype=F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, dtype=F64)


def rope(v, pos, theta):
    """Rotary embedding with half-split pairing: element i is paired with i + D/2 and the pair
    is rotated by angle pos * theta^(-2i/D). v: [..., n, H, D], pos: [n]."""
    if not theta:
        return np.asarray(v, dtype=F64)
    v = np.asarray(v, dtype=F64)
    D = v.shape[-1]
    half = D // 2
    inv_freq = F64(theta) ** (-np.arange(half, dtype=F64) * 2.0 / D)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv_freq[None, :]      # [n, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def tree_attention(q, k_new, v_new, K, V, anc):
    """q: [n, Hq, D]; k_new, v_new: [n, Hkv, D]; K, V: [Hkv, L, D] (prefix cache); anc: [n, n].
    Node i, head h attends to every cache position and to the tree nodes j with anc[i, j];
    logits scaled by 1/sqrt(D); softmax; weighted sum of values. Returns [n, Hq, D]."""
    q = np.asarray(q, F64); k_new = np.asarray(k_new, F64); v_new = np.asarray(v_new, F64)
    K = np.asarray(K, F64); V = np.asarray(V, F64)
    n, Hq, D = q.shape
    Hkv = K.shape[0]
    group = Hq // Hkv
    out = np.zeros((n, Hq, D), dtype=F64)
    scale = 1.0 / np.sqrt(F64(D))
    for i in range(n):
        vis = np.nonzero(anc[i])[0]
        for h in range(Hq):
            g = h // group
            keys = np.concatenate([K[g], k_new[vis, g]], axis=0)       # [L + |path|, D]
            vals = np.concatenate([V[g], v_new[vis, g]], axis=0)
            s = keys @ q[i, h] * scale
            s = s - s.max()
            p = np.exp(s)
            p = p / p.sum()
            out[i, h] = p @ vals
    return out


def router_topk(h_norm, wg, k, norm="softmax"):
    """Eq. 4: scores W_g h, indices of the k largest (ordered by value descending, index
    ascending on equal values), selected scores normalised into weights: by softmax over the
    selected scores, or ("sigmoid", the other choice Sec. 2.2 names) by the sigmoid of each
    divided by the sum of the k sigmoids. Scores are formed in float64 and stored as float32;
    the selection is taken on the float32 values."""
    logits = (np.asarray(h_norm, F64) @ np.asarray(wg, F64).T).astype(F32)
    n, E = logits.shape
    idx = np.zeros((n, k), dtype=np.int32)
    w = np.zeros((n, k), dtype=F32)
    for t in range(n):
        order = sorted(range(E), key=lambda e: (-float(logits[t, e]), e))[:k]
        idx[t] = order
        s = logits[t, order].astype(F64)
        p = 1.0 / (1.0 + np.exp(-s)) if norm == "sigmoid" else np.exp(s - s.max())
        w[t] = (p / p.sum()).astype(F32)
    return idx, w, logits


def router_margin(logits, k):
    """Gap between the k-th and (k+1)-th largest score of each token."""
    srt = -np.sort(-np.asarray(logits, F64), axis=-1)
    if srt.shape[-1] <= k:
        return np.full(srt.shape[0], np.inf)
    return srt[:, k - 1] - srt[:, k]


def expert_union(idx, E):
    """Eq. 5 and the grouping it induces: hist[e] = number of (token, slot) pairs routed to e;
    union = experts with hist > 0 in ascending order; offsets = exclusive prefix sum of hist;
    perm lists pair ids (token * k + slot) grouped by expert, ascending pair id within an
    expert; inv[token, slot] is the position of that pair in perm."""
    idx = np.asarray(idx)
    n, k = idx.shape
    hist = np.zeros(E, dtype=np.int32)
    for t in range(n):
        for j in range(k):
            hist[idx[t, j]] += 1
    union = np.asarray([e for e in range(E) if hist[e] > 0], dtype=np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offsets[e + 1] = offsets[e] + hist[e]
    perm = np.zeros(n * k, dtype=np.int32)
    inv = np.zeros((n, k), dtype=np.int32)
    fill = offsets[:-1].copy()
    for t in range(n):
        for j in range(k):
            e = idx[t, j]
            perm[fill[e]] = t * k + j
            inv[t, j] = fill[e]
            fill[e] += 1
    return {"union_ids": union, "union_count": int(len(union)), "hist": hist,
            "offsets": offsets, "perm": perm, "inv": inv}


def silu(z):
    return z / (1.0 + np.exp(-z))


def expert_mlp(x, w_gate, w_up, w_down, act):
    """SiLU-gated MLP of one expert on rows x: W_down (SiLU(W_gate x) * (W_up x))."""
    x = np.asarray(x, F64)
    a = silu(x @ np.asarray(w_gate, F64).T) * (x @ np.asarray(w_up, F64).T)
    a = handoff(a, act)
    return a @ np.asarray(w_down, F64).T


def moe_experts(h_norm, idx, W, act):
    """y[t, j] = expert idx[t, j] applied to h_norm[t] (not yet weighted). Evaluated expert by
    expert over the union, each expert on the tokens routed to it."""
    n, k = idx.shape
    d = h_norm.shape[1]
    y = np.zeros((n, k, d), dtype=F64)
    for e in np.unique(idx):
        tt, jj = np.nonzero(idx == e)
        y[tt, jj] = expert_mlp(h_norm[tt], W["w_gate"][e], W["w_up"][e], W["w_down"][e], act)
    return y


def moe_combine(h, y, w, shared=None):
    """out = h + sum_j w[t, j] * y[t, j] in slot order j = 0..k-1, then shared experts."""
    out = np.asarray(h, F64).copy()
    for j in range(y.shape[1]):
        out = out + np.asarray(w, F64)[:, j:j + 1] * y[:, j]
    if shared is not None:
        out = out + shared
    return out


# --------------------------------------------------------------------------------------
# one decoder layer over a batch of trees
# --------------------------------------------------------------------------------------
def verify_layer(cfg, W, tree_off, parent, x, K_list, V_list, ctx_len, act=None):
    """Verify all nodes of every tree in one pass through one MoE decoder layer.

    tree_off: int[B+1]; parent: tree-local parents concatenated; x: [T, d]; K_list/V_list:
    per-sequence caches [Hkv, L_b, D]; ctx_len: int[B]. `act` selects the storage type of
    activations between stages (defaults to cfg.dtype). Returns every intermediate."""
    act = act or cfg.dtype
    T = x.shape[0]
    B = len(tree_off) - 1
    x = np.asarray(x, F64)
    xn = handoff(rmsnorm(x, W["g_attn"], cfg.eps), act)
    q = (xn @ np.asarray(W["wq"], F64).T).reshape(T, cfg.Hq, cfg.D)
    kn = (xn @ np.asarray(W["wk"], F64).T).reshape(T, cfg.Hkv, cfg.D)
    vn = (xn @ np.asarray(W["wv"], F64).T).reshape(T, cfg.Hkv, cfg.D)
    o = np.zeros((T, cfg.Hq, cfg.D), dtype=F64)
    depth_all = np.zeros(T, dtype=np.int64)
    for b in range(B):
        lo, hi = int(tree_off[b]), int(tree_off[b + 1])
        anc, depth = tree_ancestors(parent[lo:hi])
        depth_all[lo:hi] = depth
        pos = int(ctx_len[b]) + depth
        q[lo:hi] = rope(q[lo:hi], pos, cfg.theta)
        kn[lo:hi] = rope(kn[lo:hi], pos, cfg.theta)
    q = handoff(q, act); kn = handoff(kn, act); vn = handoff(vn, act)
    for b in range(B):
        lo, hi = int(tree_off[b]), int(tree_off[b + 1])
        anc, _ = tree_ancestors(parent[lo:hi])
        L = int(ctx_len[b])
        o[lo:hi] = tree_attention(q[lo:hi], kn[lo:hi], vn[lo:hi],
                                  np.asarray(K_list[b])[:, :L], np.asarray(V_list[b])[:, :L], anc)
    o = handoff(o, act)
    h = handoff(x + o.reshape(T, -1) @ np.asarray(W["wo"], F64).T, act)
    res = {"x_norm": xn, "q": q, "k_new": kn, "v_new": vn, "o": o, "h": h, "depth": depth_all}
    res.update(moe_block(cfg, W, h, act))
    return res


def moe_block(cfg, W, h, act=None):
    """Router, union, experts and combine on the post-attention hidden states h [T, d]."""
    act = act or cfg.dtype
    hn = handoff(rmsnorm(h, W["g_moe"], cfg.eps), act)
    res = {"h_norm": hn}
    res.update(moe_from_normed(cfg, W, h, hn, act))
    return res


def moe_from_normed(cfg, W, h, hn, act=None):
    act = act or cfg.dtype
    idx, w, logits = router_topk(hn, W["wg"], cfg.k, getattr(cfg, "router_norm", "softmax"))
    un = expert_union(idx, cfg.E)
    y = moe_experts(hn, idx, W, act)
    shared = None
    if cfg.n_shared:
        shared = np.zeros_like(np.asarray(h, F64))
        for s in range(cfg.n_shared):
            shared = shared + expert_mlp(hn, W["ws_gate"][s], W["ws_up"][s], W["ws_down"][s], act)
    out = handoff(moe_combine(h, y, w, shared), act)
    res = {"topk_idx": idx, "topk_w": w, "router_logits": logits, "y": y, "out": out}
    res.update(un)
    return res


def lm_head_argmax(x, gain, w_lm, eps, act="f32"):
    """Final norm, logits = W_lm x, next token = argmax (lowest index on equal values)."""
    xn = handoff(rmsnorm(x, gain, eps), act)
    logits = (xn @ np.asarray(w_lm, F64).T).astype(F32)
    return np.argmax(logits, axis=-1).astype(np.int32), logits


# --------------------------------------------------------------------------------------
# greedy acceptance (temperature-0 case of the sibling rule, Sec. 2.1)
# --------------------------------------------------------------------------------------
def accept_path(parent, draft_tok, target_next):
    """Walk from the root: at node u the target's token is target_next[u]; the first child of
    u (ascending index) carrying that token is accepted and the walk continues from it; the
    walk stops when no child matches. The root is always accepted (it was sampled from the
    target). Returns (path node ids, bonus token = target_next[last accepted])."""
    n = len(parent)
    cur = 0
    path = [0]
    while True:
        nxt = None
        for c in range(cur + 1, n):
            if parent[c] == cur and draft_tok[c] == target_next[cur]:
                nxt = c
                break
        if nxt is None:
            break
        cur = nxt
        path.append(cur)
    return np.asarray(path, dtype=np.int32), int(target_next[cur])


# --------------------------------------------------------------------------------------
# acceptance under sampling: the sequential sibling rule (Sec. 2.1, Eq. 3)
# --------------------------------------------------------------------------------------
def softmax_temperature(logits, temperature):
    """Target distribution of every node: softmax(logits / temperature), float64."""
    z = np.asarray(logits, F64) / F64(temperature)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def accept_path_sampled(parent, draft_tok, P, u_node, u_bonus, with_trace=False):
    """Tree verification under sampling (Sec. 2.1, Eq. 3).

    P[u] is the target distribution over the vocabulary after node u; u_node[c] in [0, 1) is
    the random number spent when child c is tried, u_bonus the one spent on the final draw.
    At the surviving node u the children are tried in ascending index: c is accepted with
    the current probability of its token; on rejection that token's mass is set to zero and
    the rest is divided by (1 - that mass) (Eq. 3), then the next sibling is tried. When a
    child is accepted the walk moves to it with that child's own (fresh) distribution. When no
    child is left, one token is drawn from the current distribution by inverting its
    cumulative sum at u_bonus (smallest token whose cumulative mass exceeds u_bonus).
    Returns (path node ids, bonus token[, trace of (child, probability used, accepted)])."""
    n = len(parent)
    cur = 0
    path = [0]
    trace = []
    while True:
        p = np.array(P[cur], dtype=F64)
        nxt = None
        for c in range(cur + 1, n):
            if parent[c] != cur:
                continue
            pc = p[draft_tok[c]]
            ok = bool(u_node[c] < pc)
            trace.append((c, float(pc), ok))
            if ok:
                nxt = c
                break
            p[draft_tok[c]] = 0.0
            p = p / (1.0 - pc)
        if nxt is None:
            cdf = np.cumsum(p)
            # (the last entry of the cumulative sum may fall short of 1 by rounding)
            tok = int(min(np.searchsorted(cdf, F64(u_bonus) * cdf[-1], side="right"), len(p) - 1))
            if with_trace:
                return np.asarray(path, dtype=np.int32), tok, trace, cdf / cdf[-1]
            return np.asarray(path, dtype=np.int32), tok
        cur = nxt
        path.append(cur)


def kv_commit(K, V, k_new, v_new, path):
    """What follows acceptance in one sequence: the keys / values of the accepted path's nodes
    (rows of k_new / v_new [n, Hkv, D], already rotated at context_length + depth) are appended
    to the cache [Hkv, L, D] in path order, so the j-th accepted node (depth j) lands at
    position L + j. Returns the extended (K, V)."""
    kn = np.asarray(k_new)[np.asarray(path)]          # [len, Hkv, D]
    vn = np.asarray(v_new)[np.asarray(path)]
    return (np.concatenate([np.asarray(K), np.transpose(kn, (1, 0, 2))], axis=1),
            np.concatenate([np.asarray(V), np.transpose(vn, (1, 0, 2))], axis=1))


def paged_view(pool, table_row, L, page_size):
    """A sequence's cache [Hkv, L, D] read out of a page pool [n_pages, Hkv, page_size, D]:
    position p is row p mod page_size of page table_row[p div page_size] (the block-table layout
    of serving engines; a storage layout, not part of the method's arithmetic)."""
    pool = np.asarray(pool)
    out = np.empty((pool.shape[1], L, pool.shape[3]), dtype=pool.dtype)
    for p in range(L):
        out[:, p, :] = pool[int(table_row[p // page_size]), :, p % page_size, :]
    return out


def kv_commit_paged(pool_k, pool_v, table_row, L, k_new, v_new, path, page_size):
    """kv_commit on a paged cache, in place: the j-th accepted node goes to position L + j, i.e.
    row (L + j) mod page_size of page table_row[(L + j) div page_size]. Returns the new length."""
    for j, node in enumerate(path):
        p = L + j
        pg, r = int(table_row[p // page_size]), p % page_size
        pool_k[pg, :, r, :] = np.asarray(k_new)[node]
        pool_v[pg, :, r, :] = np.asarray(v_new)[node]
    return L + len(path)


# --------------------------------------------------------------------------------------
# EVICT prefix selection (Sec. 3.1-3.2)
# --------------------------------------------------------------------------------------
def node_scores(parent, q):
    """Eq. 7 in float32: Score(root) = 1, Score(v) = Score(parent(v)) * q(v), one rounded
    multiply per node in ascending node order."""
    n = len(parent)
    s = np.zeros(n, dtype=F32)
    s[0] = F32(1.0)
    for i in range(1, n):
        s[i] = F32(s[parent[i]]) * F32(q[i])
    return s


def select_prefix(parent, q, cost, kmax):
    """Rank nodes by score (descending, lower index first on ties: with parent[i] < i every
    prefix is then ancestor-closed, Sec. 3.2.1); S_k = running float32 sum of the k best
    scores (Eq. 8 on T_k); u_k = S_k / cost[k] in float32; k* = smallest k in
    1..min(N, kmax) attaining max u_k (Eq. 10). cost[0] is unused."""
    n = len(parent)
    score = node_scores(parent, q)
    order = np.asarray(sorted(range(n), key=lambda i: (-float(score[i]), i)), dtype=np.int32)
    kk = min(n, int(kmax))
    S = np.zeros(kk, dtype=F32)
    u = np.zeros(kk, dtype=F32)
    acc = F32(0.0)
    for j in range(kk):
        acc = F32(acc + score[order[j]])
        S[j] = acc
        u[j] = F32(acc / F32(cost[j + 1]))
    kstar = 1
    best = u[0]
    for j in range(1, kk):
        if u[j] > best:
            best = u[j]
            kstar = j + 1
    keep = np.sort(order[:kstar]).astype(np.int32)
    rank = {int(v): r for r, v in enumerate(keep)}
    new_parent = np.asarray([-1 if parent[v] < 0 else rank[int(parent[v])] for v in keep],
                            dtype=np.int32)
    su = np.sort(u.astype(F64))[::-1]
    margin = float(su[0] - su[1]) if kk > 1 else float("inf")
    return {"k_star": kstar, "order": order, "score": score, "S": S, "u": u, "keep": keep,
            "new_parent": new_parent, "est_len": F32(S[kstar - 1]), "margin": margin}


def select_prefix_coverage(parent, q, rho, kmax):
    """Cost-agnostic ablation (Sec. 4.3.2): same ranking and float32 running sums as
    select_prefix; k* = smallest k in 1..min(N, kmax) with S_k / S_N >= rho (float32 division),
    or the whole budget when no such k exists."""
    n = len(parent)
    score = node_scores(parent, q)
    order = np.asarray(sorted(range(n), key=lambda i: (-float(score[i]), i)), dtype=np.int32)
    S = np.zeros(n, dtype=F32)
    acc = F32(0.0)
    for j in range(n):
        acc = F32(acc + score[order[j]])
        S[j] = acc
    kk = min(n, int(kmax))
    kstar = kk
    for j in range(kk):
        if F32(S[j] / S[n - 1]) >= F32(rho):
            kstar = j + 1
            break
    keep = np.sort(order[:kstar]).astype(np.int32)
    rank = {int(v): r for r, v in enumerate(keep)}
    new_parent = np.asarray([-1 if parent[v] < 0 else rank[int(parent[v])] for v in keep], dtype=np.int32)
    return {"k_star": kstar, "order": order, "S": S, "keep": keep, "new_parent": new_parent, "est_len": F32(S[kstar - 1])}


def expected_accept_len_exact(parent, p):
    """Eq. 6: sum over nodes of the product of acceptance probabilities along the root path."""
    n = len(parent)
    path = np.zeros(n, dtype=F64)
    for i in range(n):
        path[i] = F64(p[i]) * (path[parent[i]] if parent[i] >= 0 else 1.0)
    return float(path.sum())


def expected_unique_experts(M, K, t):
    """App. A, Eq. 11: M * (1 - (1 - K/M)^t)."""
    return M * (1.0 - (1.0 - K / M) ** t)
