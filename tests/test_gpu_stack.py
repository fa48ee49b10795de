"""GPU parity of the multi-layer pass, the LM head + argmax, the whole selection -> verification ->
acceptance pipeline on truncated trees, and the on-device cost profile, against the CPU oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle import evict_oracle as orc

pytestmark = pytest.mark.gpu

ev = pytest.importorskip("paper_2605_00342_amd")
from paper_2605_00342_amd import harness  # noqa: E402

from tolerances import TOL, stack_tol  # noqa: E402

DEV = "cuda:0"


def rel_l2(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-30))


def make_stack(cfg_name, n_layers, n, L, seed, batch=1, L_list=None, tree="auto"):
    case = synth.make_case(cfg_name, n=n, L=L, seed=seed, batch=batch, L_list=L_list, tree=tree)
    cfg = case["cfg"]
    Ws = [case["W"]] + [synth.layer_weights(cfg, synth.philox(seed, 1000 + l)) for l in range(1, n_layers)]
    Ks, Vs = [case["K"]], [case["V"]]
    for l in range(1, n_layers):
        kv = [synth.kv_cache(cfg, int(Lb), synth.philox(seed, 2000 + 10 * l + b)) for b, Lb in enumerate(case["ctx_len"])]
        Ks.append([k for k, _ in kv]); Vs.append([v for _, v in kv])
    return case, Ws, Ks, Vs


class DeviceStack:
    def __init__(self, case, Ws, Ks, Vs, vocab=0, max_tokens=None):
        cfg = case["cfg"]
        T = int(case["tree_off"][-1])
        self.cfg, self.T, self.B = cfg, T, len(case["ctx_len"])
        self.layers = [harness.DeviceLayer(cfg, Ws[0], max_tokens or T, self.B, int(max(case["ctx_len"])), vocab=vocab)]
        self.ctx = self.layers[0].ctx
        for W in Ws[1:]:
            self.layers.append(harness.DeviceLayer(cfg, W, 0, 0, 0, ctx=self.ctx))
        self.cases = []
        for l in range(len(Ws)):
            c = dict(case); c["K"], c["V"] = Ks[l], Vs[l]
            self.cases.append(harness.DeviceCase(c, with_aux=False))
        self.dc = self.cases[0]

    def run(self, tree_off=None, parent=None, T=None, x=None, out=None):
        dc = self.dc
        ev.evict_verify_stack(self.ctx, [l.weights for l in self.layers], tree_off if tree_off is not None else dc.tree_off,
                              parent if parent is not None else dc.parent, self.B, T or self.T,
                              [c.k_cache for c in self.cases], [c.v_cache for c in self.cases], dc.seq_stride, dc.head_stride,
                              dc.ctx_len, dc.max_ctx, x if x is not None else dc.x, out if out is not None else dc.out,
                              [c.k_new for c in self.cases], [c.v_new for c in self.cases])

    def close(self):
        self.layers[0].close()


def oracle_stack(case, Ws, Ks, Vs, tree_off=None, parent=None, x=None):
    cfg = case["cfg"]
    x = case["x"] if x is None else x
    outs = []
    for l in range(len(Ws)):
        r = orc.verify_layer(cfg, Ws[l], case["tree_off"] if tree_off is None else tree_off,
                             case["parent"] if parent is None else parent, x, Ks[l], Vs[l], case["ctx_len"])
        outs.append(r)
        x = r["out"]
    return outs


@pytest.mark.parametrize("cfg_name,n,L,seed", [("tiny", 9, 40, 40), ("mini_bf16", 20, 70, 41)])
def test_stack_of_layers_matches_oracle(cfg_name, n, L, seed):
    case, Ws, Ks, Vs = make_stack(cfg_name, 3, n, L, seed)
    st = DeviceStack(case, Ws, Ks, Vs)
    ev.evict_union_total(st.ctx, reset=True)
    st.run()
    torch.cuda.synchronize()
    ref = oracle_stack(case, Ws, Ks, Vs)
    assert rel_l2(harness.to_host(st.dc.out), ref[-1]["out"]) < stack_tol(case["cfg"].dtype, 3)
    # the running total of |union| (Eq. 5) over the three layer passes: the oracle's routing, up to one near-tie flip per layer
    total = ev.evict_union_total(st.ctx, reset=True)
    assert abs(total - sum(int(r["union_count"]) for r in ref)) <= 3
    assert ev.evict_union_total(st.ctx) == 0  # the read above cleared it
    for l in range(3):
        assert rel_l2(harness.to_host(st.cases[l].k_new), ref[l]["k_new"]) < stack_tol(case["cfg"].dtype, l + 1)
    assert ev.evict_device_status(st.ctx) == 0
    # the stack equals the same layers called one by one
    x = st.dc.x
    for l in range(3):
        o = torch.zeros_like(st.dc.out)
        c = st.cases[l]
        ev.evict_verify_layer(st.ctx, st.layers[l].weights, c.tree_off, c.parent, 1, n, c.k_cache, c.v_cache, c.seq_stride,
                              c.head_stride, c.ctx_len, c.max_ctx, x, o, c.k_new, c.v_new, None)
        x = o
    torch.cuda.synchronize()
    assert torch.equal(x, st.dc.out)
    st.close()


@pytest.mark.parametrize("cfg_name,vocab,T,seed", [("tiny", 1008, 8, 50), ("mini_bf16", 4000, 37, 51), ("mini_bf16", 160, 1, 52),
                                                  ("tiny", 1008, 40, 53), ("mini_bf16", 4000, 100, 54), ("mini_bf16", 48, 17, 55)])
def test_lm_head_argmax_matches_oracle(cfg_name, vocab, T, seed):
    cfg = synth.CONFIGS[cfg_name]
    g = synth.philox(seed, 1)
    x = synth.store(g.standard_normal((T, cfg.d)), cfg.dtype)
    gain = synth.store(1.0 + 0.1 * g.standard_normal(cfg.d), cfg.dtype)
    w_lm = synth.store(g.standard_normal((vocab, cfg.d)) * 0.05, cfg.dtype)
    if T > 4:
        w_lm[7] = w_lm[3]            # two identical rows: equal logits must go to the lower index
    ctx = ev.evict_create(harness.model_desc(cfg, vocab), T, 1, 16)
    wp = harness.pack_lm_head(cfg, w_lm)
    nxt = torch.zeros(T, dtype=torch.int32, device=DEV)
    best = torch.zeros(T, device=DEV)
    xd, gd = harness.to_dev(x, cfg.dtype), harness.to_dev(gain, cfg.dtype)
    xn = torch.zeros_like(xd)
    ev.evict_lm_head_argmax(ctx, xd, gd, wp, T, nxt, best, xn)
    torch.cuda.synchronize()
    # stage-wise: logits from the normalised input the GPU used; near-ties excluded and counted
    logits = (np.asarray(harness.to_host(xn), np.float64) @ np.asarray(w_lm, np.float64).T).astype(np.float32)
    srt = -np.sort(-logits.astype(np.float64), axis=-1)
    uniq_gap = np.array([np.min(np.diff(np.unique(-row))[:1]) if len(np.unique(row)) > 1 else np.inf for row in logits])
    ok = uniq_gap >= 1e-4
    assert (~ok).sum() <= max(1, T // 8)
    ref = np.argmax(logits, axis=-1)     # first (lowest) index on equal values
    assert np.array_equal(nxt.cpu().numpy()[ok], ref[ok])
    np.testing.assert_allclose(best.cpu().numpy(), logits.max(-1), rtol=0, atol=2e-5)
    # end to end against the oracle's own normalisation
    ref2, _ = orc.lm_head_argmax(x, gain, w_lm, cfg.eps, act=cfg.dtype)
    assert rel_l2(harness.to_host(xn), orc.handoff(orc.rmsnorm(x, gain, cfg.eps), cfg.dtype)) < TOL[cfg.dtype]
    assert (ref2 != nxt.cpu().numpy()).sum() <= max(1, T // 8)
    ev.evict_destroy(ctx)


def test_select_verify_lmhead_accept_pipeline_on_truncated_trees():
    """EVICT selection first, the truncated trees verified in one batched pass, greedy acceptance
    on the target's tokens: every step against the oracle fed with the previous GPU step."""
    cfg_name, vocab, seed = "mini_bf16", 512, 60
    case, Ws, Ks, Vs = make_stack(cfg_name, 2, 24, 0, seed, batch=3, L_list=[33, 70, 5], tree="bfs")
    cfg = case["cfg"]
    T, B = int(case["tree_off"][-1]), 3
    st = DeviceStack(case, Ws, Ks, Vs, vocab=vocab)
    i32 = torch.int32
    cost = synth.cost_linear_in_union(24, cfg.E, cfg.k, a=1.0, b=0.4)
    ks = torch.zeros(B, dtype=i32, device=DEV); keep = torch.zeros(T, dtype=i32, device=DEV)
    npar = torch.zeros(T, dtype=i32, device=DEV); noff = torch.zeros(B + 1, dtype=i32, device=DEV); est = torch.zeros(B, device=DEV)
    ev.evict_select_prefix(None, st.dc.tree_off, st.dc.parent, torch.from_numpy(case["q"]).to(DEV), B, T,
                           torch.from_numpy(cost).to(DEV), 24, ks, keep, npar, noff, est)
    x2 = torch.zeros_like(st.dc.x)
    eb = 2
    ev.evict_gather_rows(st.dc.x, x2, cfg.d * eb, st.dc.tree_off, noff, keep, B, T)
    torch.cuda.synchronize()
    noff_h, keep_h, npar_h = noff.cpu().numpy(), keep.cpu().numpy(), npar.cpu().numpy()
    T2 = int(noff_h[B])
    # oracle selection
    xs, pars = [], []
    for b in range(B):
        lo, hi = case["tree_off"][b], case["tree_off"][b + 1]
        ref = orc.select_prefix(case["parents"][b], case["q"][lo:hi], cost, 24)
        assert ks[b].item() == ref["k_star"]
        assert np.array_equal(keep_h[noff_h[b]:noff_h[b + 1]], ref["keep"])
        assert np.array_equal(npar_h[noff_h[b]:noff_h[b + 1]], ref["new_parent"])
        xs.append(case["x"][lo:hi][ref["keep"]]); pars.append(ref["new_parent"])
    assert 3 <= T2 < T
    x_trunc = np.concatenate(xs)
    assert np.array_equal(harness.to_host(x2)[:T2], x_trunc)
    # verify the truncated trees
    out = torch.zeros_like(st.dc.out)
    st.run(tree_off=noff, parent=npar, T=T2, x=x2, out=out)
    off2, par2 = synth.concat_trees(pars)
    ref_layers = oracle_stack(case, Ws, Ks, Vs, tree_off=off2, parent=par2, x=x_trunc)
    torch.cuda.synchronize()
    assert rel_l2(harness.to_host(out)[:T2], ref_layers[-1]["out"]) < stack_tol(cfg.dtype, 2)
    # target tokens and acceptance
    g = synth.philox(seed, 5)
    gain = synth.store(np.ones(cfg.d), cfg.dtype)
    w_lm = synth.store(g.standard_normal((vocab, cfg.d)) * 0.05, cfg.dtype)
    wp = harness.pack_lm_head(cfg, w_lm)
    nxt = torch.zeros(T, dtype=i32, device=DEV)
    ev.evict_lm_head_argmax(st.ctx, out, harness.to_dev(gain, cfg.dtype), wp, T2, nxt, None, None)
    torch.cuda.synchronize()
    nxt_h = nxt.cpu().numpy()[:T2]
    tok = np.concatenate([synth.plant_draft_tokens(pars[b], nxt_h[off2[b]:off2[b + 1]], vocab, g, 0.8) for b in range(B)]).astype(np.int32)
    path = torch.zeros(B, 16, dtype=i32, device=DEV); plen = torch.zeros(B, dtype=i32, device=DEV); bonus = torch.zeros(B, dtype=i32, device=DEV)
    ev.evict_accept_path(None, noff, npar, harness.dev_i32(tok), nxt, B, path, 16, plen, bonus)
    torch.cuda.synchronize()
    for b in range(B):
        rp, rb = orc.accept_path(pars[b], tok[off2[b]:off2[b + 1]], nxt_h[off2[b]:off2[b + 1]])
        assert plen[b].item() == len(rp) and bonus[b].item() == rb
        assert np.array_equal(path.cpu().numpy()[b, :len(rp)], rp)
    assert ev.evict_device_status(st.ctx) == 0
    st.close()


def test_profile_cost_table_and_selection_from_it():
    case, Ws, Ks, Vs = make_stack("mini_bf16", 2, 16, 64, 70)
    st = DeviceStack(case, Ws, Ks, Vs)
    dc = st.dc
    cost = ev.evict_profile_cost(st.ctx, [l.weights for l in st.layers], dc.tree_off, dc.parent, 16,
                                 [c.k_cache for c in st.cases], [c.v_cache for c in st.cases], dc.head_stride, dc.ctx_len,
                                 dc.max_ctx, dc.x, dc.out, [c.k_new for c in st.cases], [c.v_new for c in st.cases], 3)
    assert len(cost) == 17 and cost[0] == 0.0
    assert all(np.isfinite(c) and 0.0 < c < 50.0 for c in cost[1:])
    # the profiled table drives the on-device selection exactly as the oracle's
    cost_np = np.asarray(cost, np.float32); cost_np[0] = 1.0
    i32 = torch.int32
    ks = torch.zeros(1, dtype=i32, device=DEV); keep = torch.zeros(16, dtype=i32, device=DEV)
    npar = torch.zeros(16, dtype=i32, device=DEV); noff = torch.zeros(2, dtype=i32, device=DEV); est = torch.zeros(1, device=DEV)
    ev.evict_select_prefix(None, dc.tree_off, dc.parent, torch.from_numpy(case["q"]).to(DEV), 1, 16,
                           torch.from_numpy(cost_np).to(DEV), 16, ks, keep, npar, noff, est)
    torch.cuda.synchronize()
    assert ks.item() == orc.select_prefix(case["parent"], case["q"], cost_np, 16)["k_star"]
    # a prefix of the tree verified alone equals the profile's k-node case
    st.run(T=5)
    torch.cuda.synchronize()
    ref = oracle_stack(case, Ws, Ks, Vs, tree_off=np.array([0, 5], np.int32), parent=case["parent"][:5], x=case["x"][:5])
    assert rel_l2(harness.to_host(dc.out)[:5], ref[-1]["out"]) < stack_tol("bf16", 2)
    st.close()


def test_lm_head_full_vocabulary():
    # Qwen3-sized LM head: vocab 151936, d = 2048, 32 tokens
    cfg, vocab, T = synth.CONFIGS["qwen3"], 151936, 32
    g = synth.philox(80, 1)
    x = synth.store(g.standard_normal((T, cfg.d)), cfg.dtype)
    gain = synth.store(np.ones(cfg.d), cfg.dtype)
    w_lm = synth.store(g.standard_normal((vocab, cfg.d), dtype=np.float32) * np.float32(0.02), cfg.dtype)
    ctx = ev.evict_create(harness.model_desc(cfg, vocab), T, 1, 16)
    wp = harness.pack_lm_head(cfg, w_lm)
    nxt = torch.zeros(T, dtype=torch.int32, device=DEV)
    best = torch.zeros(T, device=DEV)
    xd = harness.to_dev(x, cfg.dtype)
    xn = torch.zeros_like(xd)
    ev.evict_lm_head_argmax(ctx, xd, harness.to_dev(gain, cfg.dtype), wp, T, nxt, best, xn)
    torch.cuda.synchronize()
    logits = (torch.from_numpy(harness.to_host(xn)).double() @ torch.from_numpy(w_lm).double().T).float().numpy()
    top2 = -np.sort(-logits, axis=-1)[:, :2]
    ok = (top2[:, 0] - top2[:, 1]) >= 1e-4
    assert (~ok).sum() <= 2
    assert np.array_equal(nxt.cpu().numpy()[ok], np.argmax(logits, -1)[ok])
    np.testing.assert_allclose(best.cpu().numpy(), logits.max(-1), rtol=0, atol=5e-5)
    ev.evict_destroy(ctx)


def test_profile_reports_mean_union_and_feeds_the_cost_surface():
    # two input sets of different routing spread (child noise 0.2 and 1.0) on the same weights
    from paper_2605_00342_amd import cost_model as cm
    n, L, nl = 16, 64, 2
    case, Ws, Ks, Vs = make_stack("mini_bf16", nl, n, L, 71)
    wide = synth.make_case("mini_bf16", n=n, L=L, seed=71, sigma=1.0)
    narrow = synth.make_case("mini_bf16", n=n, L=L, seed=71, sigma=0.05)
    cfg = case["cfg"]
    st = DeviceStack(case, Ws, Ks, Vs)
    dc = st.dc
    sets, refs = [], []
    for c in (narrow, wide):
        x_dev = harness.to_dev(c["x"], cfg.dtype)
        par = harness.dev_i32(c["parent"])
        sets.append(dict(tree_off=dc.tree_off, parent=par, k_caches=[q.k_cache for q in st.cases],
                         v_caches=[q.v_cache for q in st.cases], kv_head_stride=dc.head_stride, ctx_len=dc.ctx_len,
                         max_ctx_host=dc.max_ctx, x_in=x_dev, x_out=dc.out, k_new=[q.k_new for q in st.cases],
                         v_new=[q.v_new for q in st.cases]))
        # oracle: mean union over the layers for every prefix length
        means = [0.0]
        for k in range(1, n + 1):
            r = oracle_stack(dict(case, x=c["x"]), Ws, Ks, Vs, tree_off=np.array([0, k], np.int32), parent=c["parent"][:k],
                             x=c["x"][:k])
            means.append(float(np.mean([q["union_count"] for q in r])))
        refs.append(means)
    cost, umean = ev.evict_profile_cost_union(st.ctx, [l.weights for l in st.layers], sets[1]["tree_off"], sets[1]["parent"], n,
                                              sets[1]["k_caches"], sets[1]["v_caches"], dc.head_stride, dc.ctx_len, dc.max_ctx,
                                              sets[1]["x_in"], dc.out, sets[1]["k_new"], sets[1]["v_new"], 2)
    assert len(cost) == n + 1 and len(umean) == n + 1 and umean[0] == 0.0
    # the union of a single token is its k experts; means agree with the oracle's routing up to
    # one near-tie flip in one layer
    assert umean[1] == cfg.k
    assert np.max(np.abs(np.asarray(umean) - refs[1])) <= 1.0 / nl + 1e-6, (umean, refs[1])
    ks, us, ts, mean_u = cm.profile_cost_surface(st.ctx, [l.weights for l in st.layers], sets, n, 3)
    assert ks.size == 2 * n and np.all(np.isfinite(ts)) and np.all(ts > 0)
    assert np.max(np.abs(us[:n] - refs[0][1:])) <= 1.0 / nl + 1e-6 and np.max(np.abs(us[n:] - refs[1][1:])) <= 1.0 / nl + 1e-6
    assert us[n:].sum() > us[:n].sum()          # wider child noise activates more experts
    assert np.allclose(mean_u[1:], 0.5 * (us[:n] + us[n:]))
    coef, rms = cm.fit_cost_surface(ks, us, ts)
    assert np.all(np.isfinite(coef)) and np.isfinite(rms)
    # whatever the timings were, the table built from them drives the device selection as the oracle's
    table = np.maximum(coef[0] + coef[1] * np.arange(n + 1) + coef[2] * mean_u, 1e-3).astype(np.float32)
    table[0] = table[1]
    i32 = torch.int32
    ksel = torch.zeros(1, dtype=i32, device=DEV); keep = torch.zeros(n, dtype=i32, device=DEV)
    npar = torch.zeros(n, dtype=i32, device=DEV); noff = torch.zeros(2, dtype=i32, device=DEV); est = torch.zeros(1, device=DEV)
    ev.evict_select_prefix(None, dc.tree_off, dc.parent, torch.from_numpy(case["q"]).to(DEV), 1, n,
                           torch.from_numpy(table).to(DEV), n, ksel, keep, npar, noff, est)
    torch.cuda.synchronize()
    assert ksel.item() == orc.select_prefix(case["parent"], case["q"], table, n)["k_star"]
    assert ev.evict_device_status(st.ctx) == 0
    st.close()


def test_profile_prefixes_with_fp32_storage_match_oracle_routing():
    """The cost profiler verifies the first k nodes of a tree as a tree of their own (B = 1, T = k) while
    tree_off still describes the whole tree: with fp32 storage too, every prefix length must route as the
    oracle's evaluation of that prefix does (mean union per length), and a prefix call must equal the
    oracle's output for that prefix."""
    n, L, nl = 12, 48, 2
    case, Ws, Ks, Vs = make_stack("tiny", nl, n, L, 72)
    cfg = case["cfg"]
    st = DeviceStack(case, Ws, Ks, Vs)
    dc = st.dc
    refs = [0.0]
    for k in range(1, n + 1):
        r = oracle_stack(case, Ws, Ks, Vs, tree_off=np.array([0, k], np.int32), parent=case["parent"][:k], x=case["x"][:k])
        refs.append(float(np.mean([q["union_count"] for q in r])))
    cost, umean = ev.evict_profile_cost_union(st.ctx, [l.weights for l in st.layers], dc.tree_off, dc.parent, n,
                                              [c.k_cache for c in st.cases], [c.v_cache for c in st.cases], dc.head_stride,
                                              dc.ctx_len, dc.max_ctx, dc.x, dc.out, [c.k_new for c in st.cases],
                                              [c.v_new for c in st.cases], 2)
    assert umean[1] == cfg.k
    assert np.max(np.abs(np.asarray(umean) - refs)) <= 1.0 / nl + 1e-6, (umean, refs)
    # one prefix call with the full tree's offsets still in tree_off, twice: same bits, oracle's values
    for k in (5, 9):
        outs = []
        for _ in range(2):
            st.run(T=k)
            torch.cuda.synchronize()
            outs.append(dc.out[:k].clone())
        assert torch.equal(outs[0], outs[1])
        ref = oracle_stack(case, Ws, Ks, Vs, tree_off=np.array([0, k], np.int32), parent=case["parent"][:k], x=case["x"][:k])
        assert rel_l2(harness.to_host(outs[0]), ref[-1]["out"]) < TOL["f32"]
    assert ev.evict_device_status(st.ctx) == 0
    st.close()
