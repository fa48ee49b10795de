"""Pins for the layer part of the CPU oracle: brute force, library routines, invariants.

Every check compares the oracle with something other than itself: a per-node dense
evaluation of the root path written separately (oracle/brute_force.py), PyTorch CPU library
routines (scaled_dot_product_attention, topk, silu, matmul), closed forms and Monte-Carlo.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import brute_force as bf
from oracle import evict_oracle as orc


def _tiny_case(seed=0, n=8, L=64, tree="random", cfg_name="tiny"):
    return synth.make_case(cfg_name, n=n, L=L, seed=seed, tree=tree)


def _run(case, act="f64"):
    return orc.verify_layer(case["cfg"], case["W"], case["tree_off"], case["parent"], case["x"],
                            case["K"], case["V"], case["ctx_len"], act=act)


# ---------------------------------------------------------------- brute force (the benchmark spec)
@pytest.mark.parametrize("seed,tree", [(0, "random"), (1, "random"), (2, "eagle"), (3, "star")])
def test_tree_pass_equals_per_node_dense_root_path(seed, tree):
    case = _tiny_case(seed=seed, tree=tree)
    cfg = case["cfg"]
    res = _run(case)
    par = case["parent"]
    for i in range(len(par)):
        path = bf.root_path(par, i)
        out, h, top, dense_w = bf.node_output_dense(cfg, case["W"], case["x"][path],
                                                    case["K"][0], case["V"][0], int(case["ctx_len"][0]))
        assert set(int(e) for e in res["topk_idx"][i]) == top
        np.testing.assert_allclose(res["h"][i], h, rtol=0, atol=1e-9)
        np.testing.assert_allclose(res["out"][i], out, rtol=0, atol=2e-7)
        # router weights keyed by expert id
        for j, e in enumerate(res["topk_idx"][i]):
            assert abs(float(res["topk_w"][i, j]) - dense_w[e]) < 1e-6


def test_brute_force_with_shared_experts_and_mha():
    cfg = synth.ModelCfg("t_shared", "f32", d=64, Hq=4, Hkv=4, D=16, E=8, k=3, F=32, n_shared=2,
                         theta=1e4)
    case = synth.make_case("t_shared", n=6, L=10, seed=5, tree="random", cfg=cfg)
    res = _run(case)
    for i in range(6):
        path = bf.root_path(case["parent"], i)
        out, h, top, _ = bf.node_output_dense(cfg, case["W"], case["x"][path], case["K"][0],
                                              case["V"][0], 10)
        np.testing.assert_allclose(res["out"][i], out, atol=2e-7)


def test_batched_trees_equal_separate_trees():
    a = synth.make_case("tiny", n=8, L=40, seed=7, batch=2, L_list=[40, 23], tree="random")
    res = _run(a)
    for b in range(2):
        lo, hi = a["tree_off"][b], a["tree_off"][b + 1]
        single = orc.verify_layer(a["cfg"], a["W"], np.array([0, hi - lo]), a["parents"][b],
                                  a["x"][lo:hi], [a["K"][b]], [a["V"][b]], a["ctx_len"][b:b + 1],
                                  act="f64")
        np.testing.assert_allclose(res["out"][lo:hi], single["out"], atol=1e-12)


# ---------------------------------------------------------------- chain == causal decode
def test_chain_tree_equals_causal_decode_library_attention():
    case = _tiny_case(seed=11, n=6, L=20, tree="chain")
    cfg = case["cfg"]
    res = _run(case)
    L = 20
    # plain sequence: cache then the chain; library causal attention over the whole sequence
    for g in range(cfg.Hkv):
        Kseq = torch.tensor(np.concatenate([case["K"][0][g, :L], res["k_new"][:, g]]), dtype=torch.float64)
        Vseq = torch.tensor(np.concatenate([case["V"][0][g, :L], res["v_new"][:, g]]), dtype=torch.float64)
        for hh in range(g * (cfg.Hq // cfg.Hkv), (g + 1) * (cfg.Hq // cfg.Hkv)):
            Q = torch.zeros(L + 6, cfg.D, dtype=torch.float64)
            Q[L:] = torch.tensor(res["q"][:, hh])
            o = torch.nn.functional.scaled_dot_product_attention(Q[None], Kseq[None], Vseq[None],
                                                                 is_causal=True)[0, L:]
            np.testing.assert_allclose(res["o"][:, hh], o.numpy(), atol=1e-10)


def test_single_node_equals_textbook_single_query_attention():
    case = _tiny_case(seed=12, n=1, L=33)
    cfg = case["cfg"]
    res = _run(case)
    for hh in range(cfg.Hq):
        g = hh // (cfg.Hq // cfg.Hkv)
        Kc = torch.tensor(np.concatenate([case["K"][0][g], res["k_new"][:, g]]), dtype=torch.float64)
        Vc = torch.tensor(np.concatenate([case["V"][0][g], res["v_new"][:, g]]), dtype=torch.float64)
        q = torch.tensor(res["q"][:, hh])
        o = torch.nn.functional.scaled_dot_product_attention(q[None], Kc[None], Vc[None])[0]
        np.testing.assert_allclose(res["o"][:, hh], o.numpy(), atol=1e-10)


def test_tree_attention_with_explicit_mask_library():
    case = _tiny_case(seed=13, n=8, L=16)
    cfg = case["cfg"]
    res = _run(case)
    anc, _ = orc.tree_ancestors(case["parent"])
    mask = torch.tensor(np.concatenate([np.ones((8, 16), bool), anc], axis=1))
    for hh in range(cfg.Hq):
        g = hh // (cfg.Hq // cfg.Hkv)
        Kc = torch.tensor(np.concatenate([case["K"][0][g], res["k_new"][:, g]]), dtype=torch.float64)
        Vc = torch.tensor(np.concatenate([case["V"][0][g], res["v_new"][:, g]]), dtype=torch.float64)
        q = torch.tensor(res["q"][:, hh])
        o = torch.nn.functional.scaled_dot_product_attention(q[None], Kc[None], Vc[None],
                                                             attn_mask=mask[None])[0]
        np.testing.assert_allclose(res["o"][:, hh], o.numpy(), atol=1e-10)


def test_sibling_permutation_invariance():
    # star tree: swapping two leaves permutes the outputs and changes nothing else
    case = _tiny_case(seed=14, n=5, L=12, tree="star")
    res = _run(case)
    perm = np.array([0, 3, 2, 1, 4])
    res2 = orc.verify_layer(case["cfg"], case["W"], case["tree_off"], case["parent"],
                            case["x"][perm], case["K"], case["V"], case["ctx_len"], act="f64")
    np.testing.assert_allclose(res2["out"], res["out"][perm], atol=1e-12)


def test_tree_ancestors_definition():
    par = np.array([-1, 0, 0, 1, 3, 2], dtype=np.int32)
    anc, dep = orc.tree_ancestors(par)
    assert dep.tolist() == [0, 1, 1, 2, 3, 2]
    for i in range(6):
        assert set(np.nonzero(anc[i])[0]) == set(bf.root_path(par, i))


# ---------------------------------------------------------------- norm and rotary
def test_rmsnorm_unit_rms_and_scale_invariance():
    g = synth.philox(1, 1)
    x = g.standard_normal((5, 64))
    y = orc.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt((y ** 2).mean(-1)), 1.0, atol=1e-12)
    np.testing.assert_allclose(orc.rmsnorm(3.7 * x, np.ones(64), 0.0), y, atol=1e-12)
    gain = g.standard_normal(64)
    np.testing.assert_allclose(orc.rmsnorm(x, gain, 0.0), y * gain, atol=1e-12)
    # eps enters under the square root, added to the mean square
    v = np.full((1, 4), 2.0)
    np.testing.assert_allclose(orc.rmsnorm(v, np.ones(4), 5.0), v / 3.0, atol=1e-15)


def test_rope_properties():
    g = synth.philox(2, 1)
    D = 32
    q = g.standard_normal((1, 1, D))
    k = g.standard_normal((1, 1, D))
    # position 0 is the identity; norms are preserved
    np.testing.assert_allclose(orc.rope(q, [0], 1e4), q, atol=1e-15)
    np.testing.assert_allclose(np.linalg.norm(orc.rope(q, [17], 1e4)), np.linalg.norm(q), atol=1e-12)
    # inner products depend on the position difference only
    a = np.sum(orc.rope(q, [9], 1e4) * orc.rope(k, [4], 1e4))
    b = np.sum(orc.rope(q, [105], 1e4) * orc.rope(k, [100], 1e4))
    np.testing.assert_allclose(a, b, atol=1e-10)
    # complex-multiplication form of the same rotation, pairing (i, i + D/2)
    np.testing.assert_allclose(orc.rope(q, [7], 1e6)[0, 0], bf._rotate_complex(q[0, 0], 7, 1e6), atol=1e-12)
    # first pair rotates by exactly `pos` radians (frequency index 0 is 1)
    e = np.zeros((1, 1, D)); e[0, 0, 0] = 1.0
    r = orc.rope(e, [0.5], 1e4)[0, 0]
    np.testing.assert_allclose([r[0], r[D // 2]], [np.cos(0.5), np.sin(0.5)], atol=1e-15)
    # theta = 0 disables the rotation
    np.testing.assert_allclose(orc.rope(q, [5], 0), q)


# ---------------------------------------------------------------- router (Eq. 4)
def test_router_topk_against_library_topk():
    g = synth.philox(3, 1)
    hn = g.standard_normal((20, 48)).astype(np.float32)
    wg = (0.3 * g.standard_normal((32, 48))).astype(np.float32)
    idx, w, logits = orc.router_topk(hn, wg, 4)
    ref_logits = torch.tensor(hn, dtype=torch.float64) @ torch.tensor(wg, dtype=torch.float64).T
    np.testing.assert_allclose(logits, ref_logits.numpy(), rtol=1e-6, atol=1e-6)
    tv, ti = torch.topk(torch.tensor(logits), 4, dim=-1)
    assert np.array_equal(idx, ti.numpy())          # descending by value
    np.testing.assert_allclose(w.sum(-1), 1.0, atol=1e-6)
    ref_w = torch.softmax(tv.double(), dim=-1).numpy()
    np.testing.assert_allclose(w, ref_w, atol=1e-7)
    assert np.all(np.diff(w, axis=-1) <= 1e-9)       # weights follow the score order
    # softmax over the selected scores equals softmax over all scores renormalised on the set
    full = torch.softmax(torch.tensor(logits).double(), dim=-1).numpy()
    sel = np.take_along_axis(full, idx.astype(np.int64), axis=1)
    np.testing.assert_allclose(w, sel / sel.sum(-1, keepdims=True), atol=1e-7)


def test_router_sigmoid_weights_against_library():
    g = synth.philox(5, 1)
    hn = g.standard_normal((20, 48)).astype(np.float32)
    wg = (0.3 * g.standard_normal((32, 48))).astype(np.float32)
    idx, w, logits = orc.router_topk(hn, wg, 4, norm="sigmoid")
    idx0, w0, _ = orc.router_topk(hn, wg, 4)
    assert np.array_equal(idx, idx0)                 # the selection does not depend on the normalisation
    sg = torch.sigmoid(torch.tensor(np.take_along_axis(logits, idx.astype(np.int64), axis=1)).double())
    np.testing.assert_allclose(w, (sg / sg.sum(-1, keepdim=True)).numpy(), atol=1e-7)
    np.testing.assert_allclose(w.sum(-1), 1.0, atol=1e-6)
    assert not np.allclose(w, w0)                    # and differs from the softmax weights
    # the layer uses it when the config says so
    import dataclasses
    case = _tiny_case(seed=5)
    cfg2 = dataclasses.replace(case["cfg"], router_norm="sigmoid")
    a = orc.verify_layer(cfg2, case["W"], case["tree_off"], case["parent"], case["x"], case["K"], case["V"], case["ctx_len"], act="f64")
    b = _run(case)
    assert np.array_equal(a["topk_idx"], b["topk_idx"]) and not np.allclose(a["topk_w"], b["topk_w"])
    sg = 1 / (1 + np.exp(-np.take_along_axis(a["router_logits"].astype(np.float64), a["topk_idx"].astype(np.int64), axis=1)))
    np.testing.assert_allclose(a["topk_w"], sg / sg.sum(-1, keepdims=True), atol=1e-6)


def test_router_tie_break_lowest_index():
    hn = np.ones((1, 4), np.float32)
    wg = np.zeros((6, 4), np.float32)
    wg[[1, 4, 5]] = 0.5
    idx, w, _ = orc.router_topk(hn, wg, 2)
    assert idx.tolist() == [[1, 4]]
    np.testing.assert_allclose(w, [[0.5, 0.5]])


# ---------------------------------------------------------------- union (Eq. 5)
def test_expert_union_definition_and_invariants():
    g = synth.philox(4, 1)
    E, k, T = 32, 4, 19
    idx = np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    u = orc.expert_union(idx, E)
    assert u["union_ids"].tolist() == sorted(set(idx.ravel().tolist()))
    assert k <= u["union_count"] <= min(E, T * k)
    assert u["hist"].sum() == T * k
    assert sorted(u["perm"].tolist()) == list(range(T * k))
    flat = idx.ravel()
    for e in range(E):
        seg = u["perm"][u["offsets"][e]:u["offsets"][e + 1]]
        assert np.all(flat[seg] == e)
        assert np.all(np.diff(seg) > 0)             # stable: ascending pair id inside a group
    assert np.array_equal(u["perm"][u["inv"].ravel()], np.arange(T * k))


def test_identical_hidden_states_activate_exactly_k_experts():
    case = _tiny_case(seed=21, n=6, L=8)
    h = np.repeat(case["x"][:1], 6, axis=0)
    res = orc.moe_block(case["cfg"], case["W"], h, act="f64")
    assert res["union_count"] == case["cfg"].k


@pytest.mark.parametrize("M,K,t", [(128, 8, 8), (128, 8, 32), (128, 8, 64), (64, 6, 64), (256, 8, 16)])
def test_expected_unique_experts_matches_monte_carlo(M, K, t):
    g = synth.philox(5, M * 1000 + t)
    trials = 400
    tot = 0
    for _ in range(trials):
        idx = np.stack([g.permutation(M)[:K] for _ in range(t)]).astype(np.int32)
        tot += orc.expert_union(idx, M)["union_count"]
    mc = tot / trials
    assert abs(mc - orc.expected_unique_experts(M, K, t)) < 0.6
    assert orc.expected_unique_experts(M, K, 1) == pytest.approx(K)


# ---------------------------------------------------------------- experts and combine
def test_single_expert_is_a_plain_gated_mlp_library():
    case = _tiny_case(seed=22, n=5, L=8)
    cfg, W = case["cfg"], case["W"]
    hn = synth.philox(22, 9).standard_normal((5, cfg.d))
    idx = np.full((5, 1), 3, dtype=np.int32)
    y = orc.moe_experts(hn, idx, W, "f64")[:, 0]
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    ref = (torch.nn.functional.silu(t(hn) @ t(W["w_gate"][3]).T) * (t(hn) @ t(W["w_up"][3]).T)) @ t(W["w_down"][3]).T
    np.testing.assert_allclose(y, ref.numpy(), atol=1e-12)


def test_combine_linearity_and_one_hot():
    g = synth.philox(23, 1)
    h = g.standard_normal((4, 16)); y = g.standard_normal((4, 3, 16))
    w1 = g.random((4, 3)); w2 = g.random((4, 3))
    a = orc.moe_combine(h, y, w1) - h
    b = orc.moe_combine(h, y, w2) - h
    c = orc.moe_combine(h, y, 2 * w1 + 3 * w2) - h
    np.testing.assert_allclose(c, 2 * a + 3 * b, atol=1e-12)
    onehot = np.zeros((4, 3)); onehot[:, 1] = 1
    np.testing.assert_allclose(orc.moe_combine(h, y, onehot), h + y[:, 1], atol=1e-15)


def test_grouped_evaluation_equals_dense_all_experts():
    case = _tiny_case(seed=24, n=8, L=8)
    cfg, W = case["cfg"], case["W"]
    res = _run(case)
    hn = res["h_norm"]
    for t in range(8):
        for j in range(cfg.k):
            e = res["topk_idx"][t, j]
            ref = orc.expert_mlp(hn[t:t + 1], W["w_gate"][e], W["w_up"][e], W["w_down"][e], "f64")[0]
            np.testing.assert_allclose(res["y"][t, j], ref, atol=1e-13)


def test_lm_head_argmax_library():
    g = synth.philox(25, 1)
    x = g.standard_normal((7, 32)); wlm = g.standard_normal((50, 32)); gain = np.ones(32)
    nxt, logits = orc.lm_head_argmax(x, gain, wlm, 1e-6, act="f64")
    xn = x / np.sqrt((x ** 2).mean(-1, keepdims=True) + 1e-6)
    assert np.array_equal(nxt, np.argmax((xn @ wlm.T).astype(np.float32), -1))


# ---------------------------------------------------------------- storage rounding
def test_bf16_rounding_matches_library_rounding():
    g = synth.philox(26, 1)
    x = (g.standard_normal(4096) * 10 ** g.uniform(-3, 3, 4096)).astype(np.float32)
    ref = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(orc.round_bf16(x).astype(np.float32), ref)
    np.testing.assert_array_equal(synth.round_to_bf16(x), ref)
    # a tie rounds to even: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7
    assert orc.round_bf16(np.float32(1.0 + 2.0 ** -8)) == 1.0
    assert orc.round_bf16(np.float32(1.0 + 3 * 2.0 ** -8)) == 1.0 + 2.0 ** -6


def test_bf16_handoffs_stay_close_to_exact_evaluation():
    case = synth.make_case("mini_bf16", n=8, L=32, seed=3)
    exact = _run(case, act="f64")
    rounded = _run(case, act="bf16")
    rel = np.linalg.norm(rounded["out"] - exact["out"]) / np.linalg.norm(exact["out"])
    assert rel < 1e-2


# ---------------------------------------------------------------- planted mistakes are caught
def test_planted_mistakes_fail_the_pins(monkeypatch):
    """Each plausible slip, planted in the oracle on the CPU, must break the brute-force pin."""
    case = _tiny_case(seed=0)
    cfg = case["cfg"]

    def disagreement():
        res = _run(case)
        worst = 0.0
        for i in range(len(case["parent"])):
            path = bf.root_path(case["parent"], i)
            out, _, _, _ = bf.node_output_dense(cfg, case["W"], case["x"][path], case["K"][0],
                                                case["V"][0], int(case["ctx_len"][0]))
            worst = max(worst, float(np.abs(res["out"][i] - out).max()))
        return worst

    assert disagreement() < 2e-7
    real_anc = orc.tree_ancestors
    # (1) mask dropped: every node sees every tree node
    monkeypatch.setattr(orc, "tree_ancestors", lambda p: (np.ones((len(p),) * 2, bool), real_anc(p)[1]))
    assert disagreement() > 1e-4
    monkeypatch.setattr(orc, "tree_ancestors", real_anc)
    # (2) position taken as node index instead of depth
    monkeypatch.setattr(orc, "tree_ancestors", lambda p: (real_anc(p)[0], np.arange(len(p))))
    assert disagreement() > 1e-4
    monkeypatch.setattr(orc, "tree_ancestors", real_anc)
    # (3) rotation with the wrong sign
    real_rope = orc.rope
    monkeypatch.setattr(orc, "rope", lambda v, pos, th: real_rope(v, -np.asarray(pos), th))
    assert disagreement() > 1e-4
    monkeypatch.setattr(orc, "rope", real_rope)
    # (4) gate and up swapped
    real_mlp = orc.expert_mlp
    monkeypatch.setattr(orc, "expert_mlp", lambda x, g_, u_, d_, act: real_mlp(x, u_, g_, d_, act))
    assert disagreement() > 1e-5
    monkeypatch.setattr(orc, "expert_mlp", real_mlp)
    # (5) residual dropped in the combine
    real_comb = orc.moe_combine
    monkeypatch.setattr(orc, "moe_combine", lambda h, y, w, shared=None: real_comb(h, y, w, shared) - h)
    assert disagreement() > 1e-2
    monkeypatch.setattr(orc, "moe_combine", real_comb)
    # (6) softmax scale omitted
    real_att = orc.tree_attention
    monkeypatch.setattr(orc, "tree_attention",
                        lambda q, kn, vn, K, V, anc: real_att(np.asarray(q) * np.sqrt(q.shape[-1]), kn, vn, K, V, anc))
    assert disagreement() > 1e-4
    monkeypatch.setattr(orc, "tree_attention", real_att)
    assert disagreement() < 2e-7


# ---------------------------------------------------------------- KV commit between iterations
@pytest.mark.parametrize("m", [1, 3, 5])
def test_commit_then_continue_equals_one_pass(m):
    """A chain of 6 nodes verified in one pass equals: verify its first m nodes, commit them
    (depth j -> cache position L + j), then verify the remaining nodes as a chain at context
    L + m. A commit at the wrong position or with unrotated keys breaks this."""
    case = _tiny_case(seed=21, n=6, L=20, tree="chain")
    cfg, W = case["cfg"], case["W"]
    one = _run(case)
    first = orc.verify_layer(cfg, W, np.array([0, m]), case["parent"][:m], case["x"][:m], case["K"], case["V"],
                             case["ctx_len"], act="f64")
    K2, V2 = orc.kv_commit(case["K"][0], case["V"][0], first["k_new"], first["v_new"], np.arange(m))
    assert K2.shape[1] == 20 + m
    rest = orc.verify_layer(cfg, W, np.array([0, 6 - m]), np.arange(-1, 5 - m), case["x"][m:], [K2], [V2],
                            np.array([20 + m]), act="f64")
    np.testing.assert_allclose(rest["out"], one["out"][m:], rtol=0, atol=1e-9)
    np.testing.assert_allclose(rest["k_new"], one["k_new"][m:], rtol=0, atol=1e-12)


def test_commit_of_a_branch_equals_dense_root_path():
    """Commit an accepted root path of a branching tree, then decode one more token: equals the
    separately written dense evaluation of (cache + path + token) as a plain causal sequence."""
    case = _tiny_case(seed=22, n=8, L=16, tree="random")
    cfg, W = case["cfg"], case["W"]
    res = _run(case)
    leaf = 7
    path = bf.root_path(case["parent"], leaf)
    K2, V2 = orc.kv_commit(case["K"][0], case["V"][0], res["k_new"], res["v_new"], path)
    g = synth.philox(22, 77)
    xt = g.standard_normal((1, cfg.d))
    nxt = orc.verify_layer(cfg, W, np.array([0, 1]), np.array([-1]), xt, [K2], [V2], np.array([16 + len(path)]), act="f64")
    seq_x = np.concatenate([case["x"][path], xt])
    out, h, _, _ = bf.node_output_dense(cfg, W, seq_x, case["K"][0], case["V"][0], 16)
    np.testing.assert_allclose(nxt["out"][0], out, rtol=0, atol=2e-7)
