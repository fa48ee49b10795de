"""Seeded synthetic inputs shaped like the paper's MoE verification workloads.

Everything here is input preparation: random trees, hidden states correlated along
branches (the cause of expert-union growth the paper describes in Sec. 2.2), random
weights, KV caches, draft probabilities and cost vectors. All randomness comes from
numpy's counter-based Philox generator keyed by (config seed, purpose), so the CPU
oracle and the GPU path can be handed bit-identical arrays.

Values destined for bf16 storage are rounded to bf16 here (round-to-nearest-even) and
returned as float32 arrays holding bf16-representable values; `bf16_bits` gives the
16-bit patterns to upload.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import numpy as np

__all__ = [
    "ModelCfg", "CONFIGS", "philox", "round_to_bf16", "bf16_bits", "store",
    "tree_random_parents", "tree_eagle_style", "tree_bfs_random", "tree_chain", "tree_star",
    "draft_probs", "hidden_states", "layer_weights", "kv_cache", "cost_linear_in_union",
    "plant_draft_tokens", "make_case", "concat_trees", "to_pages", "stack_weights_windowed", "kv_windowed",
]


# --------------------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class ModelCfg:
    name: str
    dtype: str          # "f32" or "bf16": storage type of weights and activations
    d: int              # d_model
    Hq: int             # query heads
    Hkv: int            # KV heads
    D: int              # head_dim
    E: int              # routed experts
    k: int              # experts per token
    F: int              # expert d_ff
    n_shared: int = 0   # always-on shared experts
    eps: float = 1e-6   # RMSNorm epsilon
    theta: float = 1e6  # RoPE base (0 disables RoPE)
    w_std: float = 0.02
    router_norm: str = "softmax"  # weights of the selected scores: "softmax" or "sigmoid" (Sec. 2.2)


CONFIGS: Dict[str, ModelCfg] = {
    # tiny fp32 layer (configs[0])
    "tiny": ModelCfg("tiny", "f32", d=256, Hq=4, Hkv=2, D=64, E=16, k=2, F=128, theta=1e4),
    # Qwen3-30B-A3B-shaped layer (configs[1]); 128 experts / 8 active as in App. C.2
    "qwen3": ModelCfg("qwen3", "bf16", d=2048, Hq=32, Hkv=4, D=128, E=128, k=8, F=768),
    # DeepSeek-V2-Lite-shaped layer with plain MHA (configs[3])
    "dsv2lite": ModelCfg("dsv2lite", "bf16", d=2048, Hq=16, Hkv=16, D=128, E=64, k=6, F=1408,
                         n_shared=2, theta=1e4),
    # small bf16 shape for fast parity tests spanning several tiles with ragged tails
    "mini_bf16": ModelCfg("mini_bf16", "bf16", d=512, Hq=8, Hkv=2, D=128, E=32, k=4, F=192),
    # small shape with 256 experts / 8 active (the ratio of Ling-flash-2.0, App. C.2), sigmoid router weights, 64-wide heads
    "mini_sigmoid": ModelCfg("mini_sigmoid", "bf16", d=512, Hq=8, Hkv=4, D=64, E=256, k=8, F=128, router_norm="sigmoid"),
    # One GPU's tensor-parallel share of the paper's two larger targets (App. C.2: 128 experts / 8 active
    # served with TP=8, 256 experts / 8 active served with TP=4): the full model width and every expert,
    # with the attention heads and each expert's d_ff divided by the TP degree. The widths are those of
    # the public model cards (d_model 4096; 64 query / 4 KV heads and expert d_ff 1536 for the first,
    # 32 / 4 heads, d_ff 1024 and one shared expert for the second); a KV head is replicated where the
    # TP degree exceeds the KV head count. The layer's output is this rank's partial sum.
    "qwen3_235b_tp8": ModelCfg("qwen3_235b_tp8", "bf16", d=4096, Hq=8, Hkv=1, D=128, E=128, k=8, F=192),
    "ling_flash2_tp4": ModelCfg("ling_flash2_tp4", "bf16", d=4096, Hq=8, Hkv=1, D=128, E=256, k=8, F=256,
                                n_shared=1, router_norm="sigmoid"),
}


def philox(seed: int, purpose: int = 0) -> np.random.Generator:
    """Counter-based generator keyed by (seed, purpose)."""
    return np.random.Generator(np.random.Philox(key=[int(seed), int(purpose)]))


# --------------------------------------------------------------------------------------
# storage-dtype rounding
# --------------------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of x rounded to bf16 with round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly bf16-representable."""
    b = bf16_bits(x).astype(np.uint32) << 16
    return b.view(np.float32).reshape(np.shape(x))


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


# --------------------------------------------------------------------------------------
# trees: parent[0] = -1, parent[i] < i
# --------------------------------------------------------------------------------------
def _depths(parent: np.ndarray) -> np.ndarray:
    dep = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        dep[i] = dep[parent[i]] + 1
    return dep


def tree_random_parents(n: int, max_depth: int, g: np.random.Generator) -> np.ndarray:
    """Node i's parent uniform on 0..i-1, redrawn while it would exceed max_depth."""
    parent = np.full(n, -1, dtype=np.int32)
    dep = np.zeros(n, dtype=np.int32)
    for i in range(1, n):
        while True:
            p = int(g.integers(0, i))
            if dep[p] + 1 <= max_depth:
                break
        parent[i] = p
        dep[i] = dep[p] + 1
    return parent


def tree_eagle_style(n: int, g: np.random.Generator, first_branch: int = 4, branch: int = 2,
                     max_depth: int = 6, beta: Optional[tuple] = None):
    """Top-k style expansion: the root gets `first_branch` children, then the childless
    node of depth < max_depth with the highest cumulative draft probability (ties: lowest
    index) gets `branch` children, until n nodes exist. Returns (parent, q)."""
    parent = [-1]
    q = [1.0]
    cum = [1.0]
    dep = [0]
    has_child = [False]

    def draw():
        if beta is not None:
            return float(np.clip(g.beta(*beta), 1e-3, 1.0))
        return float(g.uniform(0.05, 1.0))

    def expand(v: int, m: int):
        has_child[v] = True
        for _ in range(m):
            if len(parent) >= n:
                return
            qq = draw()
            parent.append(v)
            q.append(qq)
            cum.append(cum[v] * qq)
            dep.append(dep[v] + 1)
            has_child.append(False)

    if n > 1:
        expand(0, first_branch)
    while len(parent) < n:
        cand = [i for i in range(len(parent)) if not has_child[i] and dep[i] < max_depth]
        if not cand:
            # every leaf is at max depth: widen the shallowest expanded node instead
            cand = [i for i in range(len(parent)) if dep[i] < max_depth]
            v = min(cand, key=lambda i: (dep[i], i))
            has_child[v] = False
        else:
            v = max(cand, key=lambda i: (cum[i], -i))
        expand(v, branch)
    return np.asarray(parent, dtype=np.int32), np.asarray(q, dtype=np.float32)


def tree_bfs_random(n: int, g: np.random.Generator, max_depth: int = 8,
                    choices=(1, 2, 3, 4)) -> np.ndarray:
    """Breadth-first growth, each node's child count drawn from `choices`."""
    parent = [-1]
    dep = [0]
    head = 0
    while len(parent) < n:
        if head >= len(parent):
            head = 0  # all leaves at max depth: go round again from the root
        if dep[head] < max_depth:
            m = int(g.choice(np.asarray(choices)))
            for _ in range(m):
                if len(parent) >= n:
                    break
                parent.append(head)
                dep.append(dep[head] + 1)
        head += 1
    return np.asarray(parent, dtype=np.int32)


def tree_chain(n: int) -> np.ndarray:
    return np.arange(-1, n - 1, dtype=np.int32)


def tree_star(n: int) -> np.ndarray:
    p = np.zeros(n, dtype=np.int32)
    p[0] = -1
    return p


def concat_trees(parents: List[np.ndarray]):
    """CSR batching: returns (tree_off int32[B+1], parent int32[T]) with tree-local parents."""
    off = np.zeros(len(parents) + 1, dtype=np.int32)
    off[1:] = np.cumsum([len(p) for p in parents])
    return off, np.concatenate(parents).astype(np.int32)


# --------------------------------------------------------------------------------------
# per-node data
# --------------------------------------------------------------------------------------
def draft_probs(n: int, g: np.random.Generator, kind: str = "uniform") -> np.ndarray:
    """Linear draft probabilities q in (0,1]; root fixed to 1."""
    if kind == "uniform":
        # the config draws log-probs as log U(0.05,1); they are exponentiated once here so
        # that both sides receive identical fp32 bits
        q = np.exp(np.log(g.uniform(0.05, 1.0, size=n))).astype(np.float32)
    elif kind == "beta22":
        q = np.clip(g.beta(2.0, 2.0, size=n), 1e-3, 1.0).astype(np.float32)
    else:
        raise ValueError(kind)
    q[0] = 1.0
    return q


def hidden_states(parent: np.ndarray, d: int, sigma: float, g: np.random.Generator,
                  dtype: str) -> np.ndarray:
    """root ~ N(0,1); child = parent + sigma * N(0,1) (correlated along branches)."""
    n = len(parent)
    x = np.zeros((n, d), dtype=np.float64)
    noise = g.standard_normal((n, d))
    x[0] = noise[0]
    for i in range(1, n):
        x[i] = x[parent[i]] + sigma * noise[i]
    return store(x, dtype)


def layer_weights(cfg: ModelCfg, g: np.random.Generator) -> Dict[str, np.ndarray]:
    """All matrices ~ N(0, w_std) in the storage dtype, contraction dimension contiguous;
    norm gains 1 + small jitter so that a dropped gain is visible to the tests."""
    s = cfg.w_std

    def w(*shape):
        return store(g.standard_normal(shape, dtype=np.float32) * np.float32(s), cfg.dtype)

    W = {
        "wq": w(cfg.Hq * cfg.D, cfg.d),
        "wk": w(cfg.Hkv * cfg.D, cfg.d),
        "wv": w(cfg.Hkv * cfg.D, cfg.d),
        "wo": w(cfg.d, cfg.Hq * cfg.D),
        "wg": w(cfg.E, cfg.d),
        "w_gate": w(cfg.E, cfg.F, cfg.d),
        "w_up": w(cfg.E, cfg.F, cfg.d),
        "w_down": w(cfg.E, cfg.d, cfg.F),
        "g_attn": store(1.0 + 0.1 * g.standard_normal(cfg.d), cfg.dtype),
        "g_moe": store(1.0 + 0.1 * g.standard_normal(cfg.d), cfg.dtype),
    }
    if cfg.n_shared:
        W["ws_gate"] = w(cfg.n_shared, cfg.F, cfg.d)
        W["ws_up"] = w(cfg.n_shared, cfg.F, cfg.d)
        W["ws_down"] = w(cfg.n_shared, cfg.d, cfg.F)
    return W


def stack_weights_windowed(cfg: ModelCfg, n_layers: int, g: np.random.Generator):
    """Weights of an n_layers-deep stack at full size without generating n_layers independent layers (620 M values
    each at the Qwen3 shape): every matrix is drawn once with n_layers - 1 extra rows (experts for the expert
    tensors), and layer l is the window [l, l + rows) of it. The layers are distinct matrices of the same
    distribution (layer l + 1 is layer l shifted by one row / one expert, with one new row / expert), each a
    zero-copy view. Returns (big, layers): the big arrays by name and the per-layer dicts of views."""
    s, x = cfg.w_std, n_layers - 1

    def w(*shape):
        return store(g.standard_normal(shape, dtype=np.float32) * np.float32(s), cfg.dtype)

    big = {
        "wq": w(cfg.Hq * cfg.D + x, cfg.d), "wk": w(cfg.Hkv * cfg.D + x, cfg.d), "wv": w(cfg.Hkv * cfg.D + x, cfg.d),
        "wo": w(cfg.d + x, cfg.Hq * cfg.D), "wg": w(cfg.E + x, cfg.d),
        "w_gate": w(cfg.E + x, cfg.F, cfg.d), "w_up": w(cfg.E + x, cfg.F, cfg.d), "w_down": w(cfg.E + x, cfg.d, cfg.F),
        "g_attn": store(1.0 + 0.1 * g.standard_normal(cfg.d + x), cfg.dtype),
        "g_moe": store(1.0 + 0.1 * g.standard_normal(cfg.d + x), cfg.dtype),
    }
    if cfg.n_shared:
        big["ws_gate"] = w(cfg.n_shared + x, cfg.F, cfg.d)
        big["ws_up"] = w(cfg.n_shared + x, cfg.F, cfg.d)
        big["ws_down"] = w(cfg.n_shared + x, cfg.d, cfg.F)
    layers = [{name: a[l:l + a.shape[0] - x] for name, a in big.items()} for l in range(n_layers)]
    return big, layers


def kv_windowed(cfg: ModelCfg, L: int, n_layers: int, g: np.random.Generator):
    """KV caches of n_layers layers for one sequence as windows over positions of one cache drawn with
    n_layers - 1 extra positions: layer l reads positions [l, l + L). Returns lists of K, V views [Hkv, L, D]."""
    K, V = kv_cache(cfg, L + n_layers - 1, g)
    return [K[:, l:l + L] for l in range(n_layers)], [V[:, l:l + L] for l in range(n_layers)]


def kv_cache(cfg: ModelCfg, L: int, g: np.random.Generator):
    """K, V ~ N(0,1), layout [Hkv, L, D]; K is taken as already position-encoded."""
    K = store(g.standard_normal((cfg.Hkv, L, cfg.D), dtype=np.float32), cfg.dtype)
    V = store(g.standard_normal((cfg.Hkv, L, cfg.D), dtype=np.float32), cfg.dtype)
    return K, V


def to_pages(Ks, Vs, page_size: int, capacities, g: np.random.Generator, spare_pages: int = 3, fill: float = 3.0e4):
    """Scatter per-sequence caches [Hkv, L_b, D] into page pools [n_pages, Hkv, page_size, D] under a
    random page assignment (pure data movement). Every sequence gets pages for capacities[b]
    positions; rows no cache position occupies, and `spare_pages` pages nobody owns, hold `fill`
    (a reader that strays shows up). Table entries past a sequence's pages hold an id outside the
    pool. Returns pool_k, pool_v, table int32 [B, max pages per sequence], n_pages."""
    B = len(Ks)
    Hkv, _, D = np.asarray(Ks[0]).shape
    need = [(int(c) + page_size - 1) // page_size for c in capacities]
    n_pages = sum(need) + spare_pages
    ids = g.permutation(n_pages)
    pool_k = np.full((n_pages, Hkv, page_size, D), fill, dtype=np.float32)
    pool_v = np.full((n_pages, Hkv, page_size, D), -fill, dtype=np.float32)
    table = np.full((B, max(max(need), 1)), n_pages + 5, dtype=np.int32)
    at = 0
    for b in range(B):
        table[b, :need[b]] = ids[at:at + need[b]]
        at += need[b]
        K, V = np.asarray(Ks[b]), np.asarray(Vs[b])
        for p in range(K.shape[1]):
            pool_k[table[b, p // page_size], :, p % page_size, :] = K[:, p, :]
            pool_v[table[b, p // page_size], :, p % page_size, :] = V[:, p, :]
    return pool_k, pool_v, table, n_pages


def cost_linear_in_union(kmax: int, E: int, k: int, a: float = 1.0, b: float = 0.05) -> np.ndarray:
    """cost[j] = a + b * U(j), U(j) the expected distinct experts for j tokens under
    independent uniform routing (App. A); cost[0] is unused and set to a."""
    j = np.arange(kmax + 1, dtype=np.float64)
    u = E * (1.0 - (1.0 - k / E) ** j)
    c = (a + b * u).astype(np.float32)
    c[0] = np.float32(a)
    return c


def plant_draft_tokens(parent: np.ndarray, target_next: np.ndarray, vocab: int,
                       g: np.random.Generator, p_match: float = 0.6) -> np.ndarray:
    """Draft token ids such that, for each node, with probability p_match its first child
    carries the target's next token; other children get distinct other ids."""
    n = len(parent)
    tok = np.zeros(n, dtype=np.int32)
    tok[0] = int(g.integers(0, vocab))
    children = [[] for _ in range(n)]
    for i in range(1, n):
        children[parent[i]].append(i)
    for v in range(n):
        ch = children[v]
        if not ch:
            continue
        nxt = int(target_next[v])
        used = {nxt}
        hit = g.random() < p_match
        for j, c in enumerate(ch):
            if j == 0 and hit:
                tok[c] = nxt
            else:
                t = int(g.integers(0, vocab))
                while t in used:
                    t = (t + 1) % vocab
                used.add(t)
                tok[c] = t
    return tok


# --------------------------------------------------------------------------------------
# whole cases
# --------------------------------------------------------------------------------------
def make_case(cfg_name: str, n: int, L: int, seed: int, sigma: Optional[float] = None,
              tree: str = "auto", batch: int = 1, L_list: Optional[List[int]] = None,
              cfg: Optional[ModelCfg] = None) -> dict:
    """One single-layer verification case: weights, batch of trees, hidden states, KV caches.

    tree: "random" (uniform parents, depth<=4), "eagle" (4 then 2, depth<=6), "bfs"
    (child counts U{1..4}, depth<=8), "chain", "star", or "auto" (the config's own recipe).
    """
    cfg = cfg or CONFIGS[cfg_name]
    if tree == "auto":
        tree = {"tiny": "random", "qwen3": "eagle", "dsv2lite": "bfs"}.get(cfg.name, "eagle")
    if sigma is None:
        sigma = 0.3 if cfg.name == "tiny" else 0.5
    W = layer_weights(cfg, philox(seed, 1))
    parents, qs, xs, Ks, Vs, Ls = [], [], [], [], [], []
    for b in range(batch):
        g = philox(seed, 100 + b)
        if tree == "random":
            par = tree_random_parents(n, 4, g)
            q = draft_probs(n, g)
        elif tree == "eagle":
            par, q = tree_eagle_style(n, g)
        elif tree == "bfs":
            par = tree_bfs_random(n, g)
            q = draft_probs(n, g, "beta22" if batch > 1 else "uniform")
        elif tree == "chain":
            par = tree_chain(n)
            q = draft_probs(n, g)
        elif tree == "star":
            par = tree_star(n)
            q = draft_probs(n, g)
        else:
            raise ValueError(tree)
        Lb = L_list[b] if L_list is not None else L
        K, V = kv_cache(cfg, Lb, philox(seed, 200 + b))
        parents.append(par)
        qs.append(q)
        xs.append(hidden_states(par, cfg.d, sigma, philox(seed, 300 + b), cfg.dtype))
        Ks.append(K)
        Vs.append(V)
        Ls.append(Lb)
    off, parent = concat_trees(parents)
    return {
        "cfg": cfg, "W": W, "tree_off": off, "parent": parent, "parents": parents,
        "q": np.concatenate(qs).astype(np.float32), "x": np.concatenate(xs, axis=0),
        "K": Ks, "V": Vs, "ctx_len": np.asarray(Ls, dtype=np.int32), "sigma": sigma,
    }
