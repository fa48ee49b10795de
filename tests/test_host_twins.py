"""Host twins of acceptance, prefix selection and expert union (no GPU): bit-exact against the CPU oracle on
seeded random inputs, the error conventions of the C ABI, and the clamp-and-flag rule for inputs the
device entry points do not trust."""
import numpy as np
import pytest

import synth
from oracle import evict_oracle as orc

ev = pytest.importorskip("paper_2605_00342_amd")


def random_tree(n, g, kind):
    if kind == "random":
        return synth.tree_random_parents(n, 6, g)
    if kind == "bfs":
        return synth.tree_bfs_random(n, g)
    if kind == "chain":
        return synth.tree_chain(n)
    return synth.tree_star(n)


@pytest.mark.parametrize("seed", range(6))
def test_select_prefix_host_equals_oracle(seed):
    g = synth.philox(seed, 77)
    parents, qs = [], []
    for b in range(int(g.integers(1, 5))):
        n = int(g.integers(1, 200))
        par = random_tree(n, g, ["random", "bfs", "chain", "star"][int(g.integers(0, 4))])
        q = synth.draft_probs(n, g, "beta22" if b % 2 else "uniform")
        q[g.random(n) < 0.1] = 1.0  # equal scores: ties go to the lower index
        parents.append(par); qs.append(q.astype(np.float32))
    off, parent = synth.concat_trees(parents)
    q = np.concatenate(qs)
    kmax = int(g.integers(1, 80))
    cost = (1.0 + 0.05 * np.arange(kmax + 1) + 0.3 * g.random(kmax + 1)).astype(np.float32)
    got = ev.evict_select_prefix_host(off, parent, q, cost, kmax)
    cov = ev.evict_select_prefix_coverage_host(off, parent, q, 0.6, kmax)
    assert got["status"] == 0 and cov["status"] == 0
    for b, par in enumerate(parents):
        lo, hi = off[b], off[b + 1]
        n = hi - lo
        for res, ref in ((got, orc.select_prefix(par, qs[b], cost, kmax)), (cov, orc.select_prefix_coverage(par, qs[b], 0.6, kmax))):
            o0, o1 = res["new_tree_off"][b], res["new_tree_off"][b + 1]
            assert res["k_star"][b] == ref["k_star"] == o1 - o0
            assert np.array_equal(res["keep"][o0:o1], ref["keep"])
            assert np.array_equal(res["new_parent"][o0:o1], ref["new_parent"])
            assert np.array_equal(res["order"][lo:hi], ref["order"])
            S = np.asarray(ref["S"], np.float32)  # (the oracle's cost rule keeps the first min(n, kmax) sums)
            assert np.array_equal(res["prefix_sum"][lo:lo + len(S)].view(np.uint32), S.view(np.uint32))
            assert np.float32(res["est_len"][b]).view(np.uint32) == np.float32(ref["est_len"]).view(np.uint32)


@pytest.mark.parametrize("seed", range(4))
def test_accept_path_host_equals_oracle(seed):
    g = synth.philox(seed, 78)
    parents, toks, nexts = [], [], []
    for b in range(3):
        n = int(g.integers(1, 150))
        par = random_tree(n, g, ["random", "bfs", "chain"][b])
        nxt = g.integers(0, 50, n).astype(np.int32)
        parents.append(par); nexts.append(nxt); toks.append(synth.plant_draft_tokens(par, nxt, 50, g, 0.8).astype(np.int32))
    off, parent = synth.concat_trees(parents)
    path, plen, bonus = ev.evict_accept_path_host(off, parent, np.concatenate(toks), np.concatenate(nexts), 8)
    for b, par in enumerate(parents):
        rp, rb = orc.accept_path(par, toks[b], nexts[b])
        assert plen[b] == len(rp) and bonus[b] == rb
        m = min(len(rp), 8)
        assert np.array_equal(path[b, :m], rp[:m]) and np.all(path[b, m:] == -1)  # longer paths: truncated, still counted


@pytest.mark.parametrize("T,k,E,seed", [(1, 2, 16, 0), (32, 8, 128, 1), (100, 6, 64, 2), (1024, 8, 256, 3)])
def test_expert_union_host_equals_oracle(T, k, E, seed):
    g = synth.philox(seed, 79)
    idx = np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    got = ev.evict_expert_union_host(idx, E)
    ref = orc.expert_union(idx, E)
    assert got["status"] == 0 and got["union_count"][0] == ref["union_count"]
    assert np.array_equal(got["union_ids"][:ref["union_count"]], ref["union_ids"]) and np.all(got["union_ids"][ref["union_count"]:] == -1)
    for name in ("hist", "offsets", "perm"):
        assert np.array_equal(got[name], ref[name]), name
    assert np.array_equal(got["inv"], np.asarray(ref["inv"]).reshape(-1))


def test_error_conventions_and_flagged_inputs():
    off = np.array([0, 4], np.int32); par = np.array([-1, 0, 0, 1], np.int32); q = np.array([1, .5, .4, .9], np.float32)
    cost = np.ones(5, np.float32)
    with pytest.raises(ev.EvictError):  # Kmax < 1
        ev.evict_select_prefix_host(off, par, q, cost, 0)
    with pytest.raises(ev.EvictError):  # rho outside [0, 1]
        ev.evict_select_prefix_coverage_host(off, par, q, 1.5, 4)
    with pytest.raises(ev.EvictError):  # k > E
        ev.evict_expert_union_host(np.zeros((2, 5), np.int32), 4)
    with pytest.raises(ev.EvictError):  # path_stride < 1
        ev.evict_accept_path_host(off, par, par, par, 0)
    # clamped and flagged, never followed: a parent that does not precede its child, a probability above 1
    # (would rank a child above its parent), a cost that is not positive (never selected), an expert id out of range
    bad = ev.evict_select_prefix_host(off, np.array([-1, 0, 3, 1], np.int32), np.array([1, .5, 1.5, np.nan], np.float32),
                                      np.array([1, 1, -1, 1, 1], np.float32), 4)
    assert bad["status"] == ev.EVICT_ST_BAD_PARENT | ev.EVICT_ST_BAD_PROB | ev.EVICT_ST_BAD_COST
    assert bad["k_star"][0] != 2  # C(2) is unusable
    ks = bad["k_star"][0]
    kept = set(bad["keep"][:ks].tolist())
    fixed_parent = [-1, 0, 0, 1]
    assert all(fixed_parent[i] < 0 or fixed_parent[i] in kept for i in kept)  # still ancestor-closed
    u = ev.evict_expert_union_host(np.array([[0, 9], [1, -3]], np.int32), 4)
    assert u["status"] == ev.EVICT_ST_BAD_EXPERT and u["hist"].sum() == 4 and u["hist"][0] == 3
