"""GPU parity of the integer / latency-bound entry points against the CPU oracle, bit-exact:
evict_select_prefix, evict_accept_path, evict_expert_union, evict_gather_rows."""
import numpy as np
import pytest
import torch

import synth
from oracle import evict_oracle as orc

pytestmark = pytest.mark.gpu

ev = pytest.importorskip("paper_2605_00342_amd")
DEV = "cuda:0"


def _i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(DEV)


def _f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV)


def _trees(sizes, seed, kind="random", maxdepth=6):
    pars, qs = [], []
    for b, n in enumerate(sizes):
        g = synth.philox(seed, 50 + b)
        if kind == "eagle":
            p, q = synth.tree_eagle_style(n, g)
        elif kind == "chain":
            p, q = synth.tree_chain(n), synth.draft_probs(n, g)
        else:
            p = synth.tree_random_parents(n, maxdepth, g)
            q = synth.draft_probs(n, g, "beta22" if b % 2 else "uniform")
        pars.append(p); qs.append(q)
    off, par = synth.concat_trees(pars)
    return off, par, pars, np.concatenate(qs).astype(np.float32), qs


def _select_gpu(off, par, q, cost, kmax):
    B, T = len(off) - 1, int(off[-1])
    d = dict(k_star=torch.zeros(B, dtype=torch.int32, device=DEV), keep=torch.full((T,), -7, dtype=torch.int32, device=DEV),
             new_parent=torch.full((T,), -7, dtype=torch.int32, device=DEV),
             new_off=torch.zeros(B + 1, dtype=torch.int32, device=DEV), est=torch.zeros(B, device=DEV),
             order=torch.zeros(T, dtype=torch.int32, device=DEV), psum=torch.zeros(T, device=DEV))
    ev.evict_select_prefix(None, _i32(off), _i32(par), _f32(q), B, T, _f32(cost), kmax, d["k_star"], d["keep"],
                           d["new_parent"], d["new_off"], d["est"], d["order"], d["psum"])
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in d.items()}


@pytest.mark.parametrize("sizes,kind,seed", [
    ([8], "random", 0), ([32], "eagle", 1), ([1], "random", 2), ([64, 64, 64, 64], "random", 3),
    ([5, 128, 1, 77, 32], "random", 4), ([200], "random", 5), ([1024], "random", 6), ([300, 1024, 17], "eagle", 7),
    ([40], "chain", 8),
])
def test_select_prefix_bit_exact(sizes, kind, seed):
    off, par, pars, q, qs = _trees(sizes, seed, kind)
    kmax = max(sizes) if seed % 2 == 0 else max(1, max(sizes) // 2)
    cost = synth.cost_linear_in_union(kmax, 128, 8)
    if seed % 3 == 1:  # a non-monotone profile
        cost = (cost * (1.0 + 0.1 * np.sin(np.arange(kmax + 1)))).astype(np.float32)
    got = _select_gpu(off, par, q, cost, kmax)
    out = 0
    for b, n in enumerate(sizes):
        ref = orc.select_prefix(pars[b], qs[b], cost, kmax)
        lo = off[b]
        assert got["k_star"][b] == ref["k_star"], (b, n)
        assert got["new_off"][b] == out
        ks = ref["k_star"]
        assert np.array_equal(got["order"][lo:lo + n], ref["order"])
        kk = min(n, kmax)
        assert np.array_equal(got["psum"][lo:lo + kk].view(np.uint32), ref["S"].view(np.uint32))   # bit-exact sums
        assert got["est"][b:b + 1].view(np.uint32)[0] == np.float32(ref["est_len"]).view(np.uint32)
        assert np.array_equal(got["keep"][out:out + ks], ref["keep"])
        assert np.array_equal(got["new_parent"][out:out + ks], ref["new_parent"])
        out += ks
    assert got["new_off"][len(sizes)] == out


def test_select_prefix_special_costs_and_ties():
    off, par, pars, q, qs = _trees([32], 11, "eagle")
    assert _select_gpu(off, par, q, np.ones(33, np.float32), 32)["k_star"][0] == 32          # constant cost
    lin = np.arange(33, dtype=np.float32); lin[0] = 1
    assert _select_gpu(off, par, q, lin, 32)["k_star"][0] == 1                               # cost = k
    q1 = np.ones(32, np.float32)                                                            # all scores tie
    got = _select_gpu(off, par, q1, np.ones(33, np.float32), 32)
    assert np.array_equal(got["order"], np.arange(32))
    ref = orc.select_prefix(pars[0], q1, lin, 32)
    assert _select_gpu(off, par, q1, lin, 32)["k_star"][0] == ref["k_star"] == 1            # u_k all equal: smallest k


@pytest.mark.parametrize("sizes,seed", [([8], 0), ([32], 1), ([1], 2), ([64, 64, 64, 64], 3), ([5, 128, 1, 77], 4),
                                        ([1024, 300], 5)])
def test_accept_path_bit_exact(sizes, seed):
    off, par, pars, _, _ = _trees(sizes, seed, "random", maxdepth=12)
    T = int(off[-1])
    g = synth.philox(seed, 60)
    nxt = g.integers(0, 1000, T).astype(np.int32)
    tok = np.concatenate([synth.plant_draft_tokens(pars[b], nxt[off[b]:off[b + 1]], 1000, g, 0.8)
                          for b in range(len(sizes))]).astype(np.int32)
    B = len(sizes)
    stride = 16
    path = torch.full((B, stride), -9, dtype=torch.int32, device=DEV)
    plen = torch.zeros(B, dtype=torch.int32, device=DEV)
    bonus = torch.zeros(B, dtype=torch.int32, device=DEV)
    ev.evict_accept_path(None, _i32(off), _i32(par), _i32(tok), _i32(nxt), B, path, stride, plen, bonus)
    torch.cuda.synchronize()
    path, plen, bonus = path.cpu().numpy(), plen.cpu().numpy(), bonus.cpu().numpy()
    for b in range(B):
        lo, hi = off[b], off[b + 1]
        rp, rb = orc.accept_path(pars[b], tok[lo:hi], nxt[lo:hi])
        assert plen[b] == len(rp) and bonus[b] == rb
        m = min(len(rp), stride)
        assert np.array_equal(path[b, :m], rp[:m]) and np.all(path[b, m:] == -1)


def test_accept_path_chain_all_match():
    n = 100
    par = synth.tree_chain(n)
    nxt = np.arange(n, dtype=np.int32) + 5
    tok = np.r_[0, nxt[:-1]].astype(np.int32)
    path = torch.zeros(1, n, dtype=torch.int32, device=DEV)
    plen = torch.zeros(1, dtype=torch.int32, device=DEV); bonus = torch.zeros(1, dtype=torch.int32, device=DEV)
    ev.evict_accept_path(None, _i32([0, n]), _i32(par), _i32(tok), _i32(nxt), 1, path, n, plen, bonus)
    torch.cuda.synchronize()
    assert plen.item() == n and bonus.item() == nxt[-1] and np.array_equal(path.cpu().numpy()[0], np.arange(n))


@pytest.mark.parametrize("T,k,E,seed", [(8, 2, 16, 0), (32, 8, 128, 1), (1, 8, 128, 2), (128, 8, 128, 3),
                                        (256, 8, 128, 4), (64, 6, 64, 5), (37, 8, 256, 6), (1024, 8, 1024, 7)])
def test_expert_union_bit_exact(T, k, E, seed):
    g = synth.philox(seed, 70)
    idx = np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    if seed == 3:
        idx[:] = idx[0]          # identical routing: union of exactly k experts
    if seed == 5:
        idx[7, 1] = idx[7, 0]    # an expert repeated inside a token: the general path must take over
        idx[20, 5] = idx[20, 2]
    ref = orc.expert_union(idx, E)
    P = T * k
    z = lambda n: torch.full((n,), -5, dtype=torch.int32, device=DEV)
    uid, uc, hist, offs, perm, inv = z(E), z(1), z(E), z(E + 1), z(P), z(P)
    ev.evict_expert_union(None, _i32(idx), T, k, E, uid, uc, hist, offs, perm, inv)
    torch.cuda.synchronize()
    U = ref["union_count"]
    assert uc.item() == U and k <= U <= min(E, T * k)
    assert np.array_equal(uid.cpu().numpy()[:U], ref["union_ids"]) and np.all(uid.cpu().numpy()[U:] == -1)
    assert np.array_equal(hist.cpu().numpy(), ref["hist"])
    assert np.array_equal(offs.cpu().numpy(), ref["offsets"])
    assert np.array_equal(perm.cpu().numpy(), ref["perm"])
    assert np.array_equal(inv.cpu().numpy(), ref["inv"].ravel())


def test_gather_rows_matches_keep_lists():
    off, par, pars, q, qs = _trees([20, 33, 7], 21, "random")
    cost = synth.cost_linear_in_union(40, 128, 8)
    got = _select_gpu(off, par, q, cost, 40)
    T = int(off[-1])
    src = torch.arange(T * 6, dtype=torch.float32, device=DEV).reshape(T, 6)
    dst = torch.full((T, 6), -1.0, device=DEV)
    d_off, d_noff, d_keep = _i32(off), _i32(got["new_off"]), _i32(got["keep"])
    ev.evict_gather_rows(src, dst, 24, d_off, d_noff, d_keep, 3, T)
    torch.cuda.synchronize()
    dst = dst.cpu().numpy(); srcn = src.cpu().numpy()
    n_new = got["new_off"][3]
    for b in range(3):
        for r in range(got["new_off"][b], got["new_off"][b + 1]):
            assert np.array_equal(dst[r], srcn[off[b] + got["keep"][r]])
    assert np.all(dst[n_new:] == -1)


@pytest.mark.parametrize("sizes,kind,seed,rho,kdiv", [
    ([32], "eagle", 1, 0.7, 1), ([32], "eagle", 1, 0.4, 1), ([1], "random", 2, 0.5, 1),
    ([64, 64, 64, 64], "random", 3, 0.85, 1), ([5, 128, 1, 77, 32], "random", 4, 1.0, 1),
    ([300, 1024, 17], "eagle", 7, 0.6, 1), ([40, 90], "random", 9, 0.999, 2), ([24], "chain", 10, 0.0, 1),
])
def test_select_prefix_coverage_bit_exact(sizes, kind, seed, rho, kdiv):
    """Cost-agnostic coverage rule (Sec. 4.3.2): smallest prefix with S_k / S_N >= rho, decided in fp32 on both sides."""
    off, par, pars, q, qs = _trees(sizes, seed, kind)
    kmax = max(1, max(sizes) // kdiv)
    B, T = len(sizes), int(off[-1])
    d = dict(k_star=torch.zeros(B, dtype=torch.int32, device=DEV), keep=torch.full((T,), -7, dtype=torch.int32, device=DEV),
             new_parent=torch.full((T,), -7, dtype=torch.int32, device=DEV),
             new_off=torch.zeros(B + 1, dtype=torch.int32, device=DEV), est=torch.zeros(B, device=DEV))
    ev.evict_select_prefix_coverage(None, _i32(off), _i32(par), _f32(q), B, T, rho, kmax, d["k_star"], d["keep"],
                                    d["new_parent"], d["new_off"], d["est"])
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in d.items()}
    out = 0
    for b, n in enumerate(sizes):
        ref = orc.select_prefix_coverage(pars[b], qs[b], rho, kmax)
        ks = ref["k_star"]
        assert got["k_star"][b] == ks, (b, n)
        assert got["new_off"][b] == out
        assert got["est"][b:b + 1].view(np.uint32)[0] == np.float32(ref["est_len"]).view(np.uint32)
        assert np.array_equal(got["keep"][out:out + ks], ref["keep"])
        assert np.array_equal(got["new_parent"][out:out + ks], ref["new_parent"])
        out += ks
    assert got["new_off"][B] == out
    with pytest.raises(ev.EvictError):
        ev.evict_select_prefix_coverage(None, _i32(off), _i32(par), _f32(q), B, T, 1.5, kmax, d["k_star"], d["keep"],
                                        d["new_parent"], d["new_off"], d["est"])


@pytest.mark.parametrize("n", [20, 100])
def test_select_prefix_flags_out_of_range_inputs_and_keeps_prefixes_closed(n):
    """A draft probability above 1 (or NaN) could rank a child above its parent; a cost entry that is not
    positive makes S_k / C(k) meaningless. Both are clamped / skipped and flagged in the context's status word,
    the result is the oracle's on the clamped inputs, and every kept node's parent is kept (Sec. 3.2.1)."""
    cfg = synth.CONFIGS["tiny"]
    from paper_2605_00342_amd import harness
    ctx = ev.evict_create(harness.model_desc(cfg), 8, 1, 16)
    off, par, pars, q, qs = _trees([n], 11, "random")
    kmax = n
    cost = synth.cost_linear_in_union(kmax, 128, 8).astype(np.float32)
    q_bad = q.copy()
    q_bad[3] = 1.75
    q_bad[7] = np.nan
    q_bad[9] = -0.25
    cost_bad = cost.copy()
    cost_bad[2] = 0.0
    cost_bad[5] = np.nan
    B, T = 1, n
    d = dict(k_star=torch.zeros(B, dtype=torch.int32, device=DEV), keep=torch.full((T,), -7, dtype=torch.int32, device=DEV),
             new_parent=torch.full((T,), -7, dtype=torch.int32, device=DEV), new_off=torch.zeros(B + 1, dtype=torch.int32, device=DEV),
             est=torch.zeros(B, device=DEV))
    # valid inputs leave the status word alone
    ev.evict_select_prefix(ctx, _i32(off), _i32(par), _f32(q), B, T, _f32(cost), kmax, d["k_star"], d["keep"], d["new_parent"],
                           d["new_off"], d["est"])
    assert ev.evict_device_status(ctx) == 0
    ev.evict_select_prefix(ctx, _i32(off), _i32(par), _f32(q_bad), B, T, _f32(cost_bad), kmax, d["k_star"], d["keep"],
                           d["new_parent"], d["new_off"], d["est"])
    st = ev.evict_device_status(ctx)
    assert st & 64 and st & 128, st
    q_fix = q_bad.copy()
    q_fix[3], q_fix[7], q_fix[9] = 1.0, 0.0, 0.0
    # the oracle on the clamped probabilities, with the unusable cost entries made so large they cannot win
    cost_fix = cost_bad.copy()
    cost_fix[2] = cost_fix[5] = np.float32(3e38)
    ref = orc.select_prefix(pars[0], q_fix, cost_fix, kmax)
    ks = int(d["k_star"][0])
    assert ks == ref["k_star"] and ks not in (2, 5)
    keep = d["keep"].cpu().numpy()[:ks]
    npar = d["new_parent"].cpu().numpy()[:ks]
    assert np.array_equal(keep, ref["keep"]) and np.array_equal(npar, ref["new_parent"])
    assert npar[0] == -1 and np.all(npar[1:] >= 0)          # one root: every kept node's parent is kept
    ev.evict_destroy(ctx)


@pytest.mark.parametrize("sizes,kind,seed", [([32], "eagle", 21), ([64, 64, 64, 64], "random", 22), ([5, 128, 1, 77, 32], "random", 23),
                                             ([300, 1024, 17], "eagle", 24)])
def test_host_twins_equal_the_device_entry_points(sizes, kind, seed):
    """evict_select_prefix_host / evict_accept_path_host / evict_expert_union_host on the host against their
    device namesakes: every output bit for bit, including the clamped-and-flagged bad inputs."""
    off, par, pars, q, qs = _trees(sizes, seed, kind)
    g = synth.philox(seed, 9)
    kmax = max(1, max(sizes) // 2)
    cost = (1.0 + 0.03 * np.arange(kmax + 1) + 0.2 * g.random(kmax + 1)).astype(np.float32)
    par_bad, q_bad = par.copy(), q.copy()
    if len(par) > 3:  # a parent that does not precede its child, a probability above 1, a NaN, an unusable cost entry
        par_bad[3] = 3; q_bad[2] = 1.5; q_bad[len(q) - 1] = np.nan
        cost[min(2, kmax)] = -1.0
    for P, Q in ((par, q), (par_bad, q_bad)):
        dev = _select_gpu(off, P, Q, cost, kmax)
        host = ev.evict_select_prefix_host(off, P, Q, cost, kmax)
        T2 = int(dev["new_off"][-1])
        assert np.array_equal(dev["k_star"], host["k_star"]) and np.array_equal(dev["new_off"], host["new_tree_off"])
        assert np.array_equal(dev["keep"][:T2], host["keep"][:T2]) and np.array_equal(dev["new_parent"][:T2], host["new_parent"][:T2])
        assert np.array_equal(dev["order"], host["order"])
        assert np.array_equal(dev["psum"].view(np.uint32), host["prefix_sum"].view(np.uint32))
        assert np.array_equal(dev["est"].view(np.uint32), host["est_len"].view(np.uint32))
    # acceptance
    B, T = len(sizes), int(off[-1])
    nxt = g.integers(0, 40, T).astype(np.int32)
    tok = np.concatenate([synth.plant_draft_tokens(p, nxt[o:o + len(p)], 40, g, 0.8) for p, o in zip(pars, off[:-1])]).astype(np.int32)
    path = torch.zeros(B, 6, dtype=torch.int32, device=DEV); plen = torch.zeros(B, dtype=torch.int32, device=DEV)
    bonus = torch.zeros(B, dtype=torch.int32, device=DEV)
    ev.evict_accept_path(None, _i32(off), _i32(par), _i32(tok), _i32(nxt), B, path, 6, plen, bonus)
    torch.cuda.synchronize()
    hp, hl, hb = ev.evict_accept_path_host(off, par, tok, nxt, 6)
    assert np.array_equal(path.cpu().numpy(), hp) and np.array_equal(plen.cpu().numpy(), hl) and np.array_equal(bonus.cpu().numpy(), hb)
    # expert union, with one expert id out of range
    E, k = 64, 6
    Tn = min(T, 8192 // k)
    idx = np.stack([g.permutation(E)[:k] for _ in range(Tn)]).astype(np.int32)
    idx[0, 0] = E + 3
    d = {n_: torch.zeros(s_, dtype=torch.int32, device=DEV) for n_, s_ in
         (("union_ids", E), ("union_count", 1), ("hist", E), ("offsets", E + 1), ("perm", Tn * k), ("inv", Tn * k))}
    ev.evict_expert_union(None, _i32(idx), Tn, k, E, d["union_ids"], d["union_count"], d["hist"], d["offsets"], d["perm"], d["inv"])
    torch.cuda.synchronize()
    hu = ev.evict_expert_union_host(idx, E)
    assert hu["status"] == ev.EVICT_ST_BAD_EXPERT
    for n_ in d:
        assert np.array_equal(d[n_].cpu().numpy(), hu[n_]), n_
