"""Several speculative iterations in a row (selection -> compaction -> layer stack -> acceptance
-> KV commit) on the GPU against the same loop composed from the CPU oracle's functions, with
the synthetic drafter's draws as shared inputs. Integers (selected length, kept nodes, accepted
path, context length) must be identical in every iteration; the hidden states of the last
iteration, which depend on every earlier commit, must agree within the layer tolerance."""
import numpy as np
import pytest
import torch

import synth
from oracle import evict_oracle as orc

pytestmark = pytest.mark.gpu

ev = pytest.importorskip("paper_2605_00342_amd")
from paper_2605_00342_amd import harness  # noqa: E402
from paper_2605_00342_amd.spec_loop import DraftOnDevice, SpecLoop  # noqa: E402

from tolerances import stack_tol  # noqa: E402

DEV = "cuda:0"


def rel_l2(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-30))


def to_device(cfg, d):
    n = len(d["parent"])
    return DraftOnDevice(harness.dev_i32(np.array([0, n])), harness.dev_i32(d["parent"]), torch.from_numpy(d["q"]).to(DEV),
                         harness.to_dev(d["x"], cfg.dtype), harness.dev_i32(d["tok"]), harness.dev_i32(d["target_next"]), n)


@pytest.mark.parametrize("cfg_name,truncate,page", [("tiny", True, 0), ("tiny", False, 0), ("mini_bf16", True, 0),
                                                    ("tiny", True, 8), ("mini_bf16", True, 16)])
def test_loop_matches_oracle_composition(cfg_name, truncate, page):
    cfg = synth.CONFIGS[cfg_name]
    n_layers, N, L0, cap, iters, seed = 2, 14, 37, 128, 4, 71
    Ws = [synth.layer_weights(cfg, synth.philox(seed, 1 + l)) for l in range(n_layers)]
    kv = [synth.kv_cache(cfg, L0, synth.philox(seed, 200 + l)) for l in range(n_layers)]
    drafts = [synth.draft_iteration(cfg, N, seed, it, 0.4, vocab=500) for it in range(iters)]
    # a cost table steep enough that truncation really cuts some trees
    cost = (1.0 + 0.35 * np.arange(N + 1)).astype(np.float32)

    layers = [harness.DeviceLayer(cfg, Ws[0], max_tokens=N, max_batch=1, max_ctx=cap)]
    for W in Ws[1:]:
        layers.append(harness.DeviceLayer(cfg, W, 0, 0, 0, ctx=layers[0].ctx))
    try:
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        kc = [torch.zeros(1, cfg.Hkv, cap, cfg.D, dtype=tdt, device=DEV) for _ in range(n_layers)]
        vc = [torch.zeros_like(k) for k in kc]
        for l in range(n_layers):
            kc[l][0, :, :L0] = harness.to_dev(kv[l][0], cfg.dtype)
            vc[l][0, :, :L0] = harness.to_dev(kv[l][1], cfg.dtype)
        if page:
            # the same caches scattered over randomly assigned pages, with pages for all `cap` positions
            pools = [synth.to_pages([kv[l][0]], [kv[l][1]], page, [cap], synth.philox(seed, 300)) for l in range(n_layers)]
            kc = [harness.to_dev(p[0], cfg.dtype) for p in pools]
            vc = [harness.to_dev(p[1], cfg.dtype) for p in pools]
            loop = SpecLoop(cfg, layers[0].ctx, [l.weights for l in layers], kc, vc, cfg.Hkv * page * cfg.D, page * cfg.D, cap, N,
                            block_table=harness.dev_i32(pools[0][2]), page_size=page, n_pages=pools[0][3])
        else:
            loop = SpecLoop(cfg, layers[0].ctx, [l.weights for l in layers], kc, vc, cfg.Hkv * cap * cfg.D, cap * cfg.D, cap, N)
        loop.set_context_length(L0)
        cost_dev = torch.from_numpy(cost).to(DEV) if truncate else None

        K = [kv[l][0] for l in range(n_layers)]
        V = [kv[l][1] for l in range(n_layers)]
        L = L0
        lens = []
        for it, d in enumerate(drafts):
            log = loop.iteration(to_device(cfg, d), cost_dev, log_lists=True)
            # ---- the same iteration from the oracle's functions
            par, x, tok, tn = d["parent"], d["x"], d["tok"], d["target_next"]
            if truncate:
                sel = orc.select_prefix(d["parent"], d["q"], cost, N)
                keep = sel["keep"]
                assert log.k_used == sel["k_star"] and log.keep == list(keep)
                par, x, tok, tn = sel["new_parent"], x[keep], tok[keep], tn[keep]
            else:
                assert log.k_used == N
            outs = []
            xin = x
            for l in range(n_layers):
                r = orc.verify_layer(cfg, Ws[l], np.array([0, len(par)]), par, xin, [K[l]], [V[l]], np.array([L]))
                outs.append(r)
                xin = r["out"]
            path, bonus = orc.accept_path(par, tok, tn)
            assert log.path == list(path) and log.bonus == bonus and log.path_len == len(path)
            for l in range(n_layers):
                K[l], V[l] = orc.kv_commit(K[l], V[l], orc.handoff(outs[l]["k_new"], cfg.dtype),
                                           orc.handoff(outs[l]["v_new"], cfg.dtype), path)
            L += len(path)
            lens.append(len(path))
            assert loop.ctx_len_host == L and int(loop.ctx_len[loop.cur].item()) == L
            tol = stack_tol(cfg.dtype, n_layers)
            assert rel_l2(harness.to_host(loop.out[: len(par)]), outs[-1]["out"]) < tol, f"iteration {it}"
        assert max(lens) > 1, "the synthetic drafter never got a token accepted: the case tests nothing"
        if truncate:
            assert ev.evict_device_status(layers[0].ctx) == 0
    finally:
        layers[0].close()


@pytest.mark.parametrize("cfg_name,truncate", [("tiny", True), ("mini_bf16", False)])
def test_loop_with_acceptance_under_sampling(cfg_name, truncate):
    """The same loop with the sequential sibling rule under sampling (Sec. 2.1, Eq. 3) on the LM head's scores.
    Draft tokens are taken from the most likely tokens under the oracle's scores of the parent (as a drafter's
    would be), so acceptances and rejections both occur. The accepted path is decided from scores computed in
    bf16 / fp32 on the GPU: the oracle's rule is applied to the GPU's own score rows (which are checked against
    the oracle's), and a decision within 1e-5 of its threshold is not compared."""
    cfg = synth.CONFIGS[cfg_name]
    n_layers, N, L0, cap, iters, seed, V, temp = 2, 14, 37, 128, 5, 73, 496, 0.8
    Ws = [synth.layer_weights(cfg, synth.philox(seed, 1 + l)) for l in range(n_layers)]
    kv = [synth.kv_cache(cfg, L0, synth.philox(seed, 200 + l)) for l in range(n_layers)]
    g = synth.philox(seed, 64)
    w_lm = synth.store((0.5 * g.standard_normal((V, cfg.d))).astype(np.float32), cfg.dtype)
    gain = synth.store((1.0 + 0.1 * g.standard_normal(cfg.d)).astype(np.float32), cfg.dtype)
    cost = (1.0 + 0.05 * np.arange(N + 1)).astype(np.float32)
    layers = [harness.DeviceLayer(cfg, Ws[0], max_tokens=N, max_batch=1, max_ctx=cap, vocab=V)]
    for W in Ws[1:]:
        layers.append(harness.DeviceLayer(cfg, W, 0, 0, 0, ctx=layers[0].ctx))
    try:
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        kc = [torch.zeros(1, cfg.Hkv, cap, cfg.D, dtype=tdt, device=DEV) for _ in range(n_layers)]
        vc = [torch.zeros_like(k) for k in kc]
        for l in range(n_layers):
            kc[l][0, :, :L0] = harness.to_dev(kv[l][0], cfg.dtype)
            vc[l][0, :, :L0] = harness.to_dev(kv[l][1], cfg.dtype)
        loop = SpecLoop(cfg, layers[0].ctx, [l.weights for l in layers], kc, vc, cfg.Hkv * cap * cfg.D, cap * cfg.D, cap, N,
                        lm_head=(harness.to_dev(gain, cfg.dtype), harness.pack_lm_head(cfg, w_lm), V))
        loop.set_context_length(L0)
        cost_dev = torch.from_numpy(cost).to(DEV) if truncate else None
        K = [kv[l][0] for l in range(n_layers)]
        Vc = [kv[l][1] for l in range(n_layers)]
        L, lens, compared = L0, [], 0
        for it in range(iters):
            d = synth.draft_iteration(cfg, N, seed, it, 0.4, vocab=V)
            par, x, q = d["parent"], d["x"], d["q"]
            keep = np.arange(N)
            if truncate:
                sel = orc.select_prefix(par, q, cost, N)
                keep, par_k = sel["keep"], sel["new_parent"]
            else:
                par_k = par
            # the oracle's layers and scores on the kept nodes (they do not depend on the dropped ones)
            outs, xin = [], x[keep]
            for l in range(n_layers):
                r = orc.verify_layer(cfg, Ws[l], np.array([0, len(par_k)]), par_k, xin, [K[l]], [Vc[l]], np.array([L]))
                outs.append(r)
                xin = r["out"]
            _, want_logits = orc.lm_head_argmax(outs[-1]["out"], gain, w_lm, cfg.eps, act=cfg.dtype)
            tok_k = np.zeros(len(par_k), np.int32)
            for u in range(len(par_k)):
                kids = [c for c in range(len(par_k)) if par_k[c] == u]
                top = np.argsort(-want_logits[u])[: max(6, len(kids))]
                order = top if g.random() < 0.6 else g.permutation(top)   # mostly the likeliest token first
                for c, t in zip(kids, order):
                    tok_k[c] = t
            tok = np.zeros(N, np.int32); tok[keep] = tok_k
            u_node = (g.random(N) ** 3).astype(np.float32)
            u_bonus = g.random(1).astype(np.float32)
            dd = DraftOnDevice(harness.dev_i32(np.array([0, N])), harness.dev_i32(par), torch.from_numpy(q).to(DEV),
                               harness.to_dev(x, cfg.dtype), harness.dev_i32(tok), None, N)
            log = loop.iteration(dd, cost_dev, log_lists=True,
                                 sample=(temp, torch.from_numpy(u_node).to(DEV), torch.from_numpy(u_bonus).to(DEV)))
            k = len(par_k)
            assert log.k_used == k and (not truncate or log.keep == list(keep))
            got_logits = loop.logits[:k].cpu().numpy()
            assert np.linalg.norm(got_logits - want_logits) / np.linalg.norm(want_logits) < stack_tol(cfg.dtype, n_layers + 1)  # (the layers, then the LM head)
            P = orc.softmax_temperature(got_logits, temp)
            rp, rb, trace, cdf = orc.accept_path_sampled(par_k, tok_k, P, u_node[keep], u_bonus[0], with_trace=True)
            if not any(abs(float(u_node[keep][c]) - p) < 1e-5 for c, p, _ in trace):
                compared += 1
                assert log.path == list(rp) and log.path_len == len(rp)
                t = log.bonus
                below = cdf[t - 1] if t > 0 else 0.0
                assert cdf[t] - below > 0.0 and below - 1e-5 <= float(u_bonus[0]) <= cdf[t] + 1e-5
            # both sides commit the path the GPU took (identical to the oracle's whenever compared)
            path = log.path
            for l in range(n_layers):
                K[l], Vc[l] = orc.kv_commit(K[l], Vc[l], orc.handoff(outs[l]["k_new"], cfg.dtype),
                                            orc.handoff(outs[l]["v_new"], cfg.dtype), path)
            L += len(path)
            lens.append(len(path))
            assert loop.ctx_len_host == L and int(loop.ctx_len[loop.cur].item()) == L
        assert compared >= iters - 1 and max(lens) > 1, (compared, lens)
        assert ev.evict_device_status(layers[0].ctx) == 0
    finally:
        layers[0].close()


class _NoReadback:
    """While active, any torch read-back to the host (.item(), .cpu(), .tolist(), .numpy()) raises."""

    NAMES = ("item", "cpu", "tolist", "numpy")

    def __enter__(self):
        self.saved = {n: getattr(torch.Tensor, n) for n in self.NAMES}

        def make(n):
            def blocked(*a, **k):
                raise AssertionError(f"host read-back through Tensor.{n}() inside the iteration")
            return blocked
        for n in self.NAMES:
            setattr(torch.Tensor, n, make(n))
        return self

    def __exit__(self, *exc):
        for n, f in self.saved.items():
            setattr(torch.Tensor, n, f)
        return False


@pytest.mark.parametrize("cfg_name,page,use_rho", [("tiny", 0, False), ("mini_bf16", 0, False), ("mini_bf16", 16, False),
                                                   ("tiny", 0, True)])
def test_loop_with_device_dispatch_reads_nothing_back_and_matches_oracle(cfg_name, page, use_rho):
    """Sec. 3.3: the selected length picks the verification without host logic in between. Every launch is sized for
    the whole draft tree, the kernels take the length from the selection's output on the device, and nothing is read
    back between selection and commit (the guard makes any read-back raise). After each iteration (outside that window)
    the logs, the accepted path, the hidden states of the kept nodes and the context length are compared with the same
    iteration composed from the oracle, exactly as for the host-dispatched loop."""
    cfg = synth.CONFIGS[cfg_name]
    n_layers, N, L0, cap, iters, seed = 2, 14, 37, 128, 5, 71
    Ws = [synth.layer_weights(cfg, synth.philox(seed, 1 + l)) for l in range(n_layers)]
    kv = [synth.kv_cache(cfg, L0, synth.philox(seed, 200 + l)) for l in range(n_layers)]
    drafts = [synth.draft_iteration(cfg, N, seed, it, 0.4, vocab=500) for it in range(iters)]
    cost = (1.0 + 0.35 * np.arange(N + 1)).astype(np.float32)
    rho = 0.6
    layers = [harness.DeviceLayer(cfg, Ws[0], max_tokens=N, max_batch=1, max_ctx=cap)]
    for W in Ws[1:]:
        layers.append(harness.DeviceLayer(cfg, W, 0, 0, 0, ctx=layers[0].ctx))
    try:
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        if page:
            pools = [synth.to_pages([kv[l][0]], [kv[l][1]], page, [cap], synth.philox(seed, 300)) for l in range(n_layers)]
            kc = [harness.to_dev(p[0], cfg.dtype) for p in pools]
            vc = [harness.to_dev(p[1], cfg.dtype) for p in pools]
            loop = SpecLoop(cfg, layers[0].ctx, [l.weights for l in layers], kc, vc, cfg.Hkv * page * cfg.D, page * cfg.D, cap, N,
                            block_table=harness.dev_i32(pools[0][2]), page_size=page, n_pages=pools[0][3])
        else:
            kc = [torch.zeros(1, cfg.Hkv, cap, cfg.D, dtype=tdt, device=DEV) for _ in range(n_layers)]
            vc = [torch.zeros_like(k) for k in kc]
            for l in range(n_layers):
                kc[l][0, :, :L0] = harness.to_dev(kv[l][0], cfg.dtype)
                vc[l][0, :, :L0] = harness.to_dev(kv[l][1], cfg.dtype)
            loop = SpecLoop(cfg, layers[0].ctx, [l.weights for l in layers], kc, vc, cfg.Hkv * cap * cfg.D, cap * cfg.D, cap, N)
        loop.set_context_length(L0)
        cost_dev = torch.from_numpy(cost).to(DEV)
        on_dev = [to_device(cfg, d) for d in drafts]
        torch.cuda.synchronize()
        K = [kv[l][0] for l in range(n_layers)]
        V = [kv[l][1] for l in range(n_layers)]
        L, lens, ks = L0, [], []
        for it, d in enumerate(drafts):
            with _NoReadback():
                slot = loop.iteration_on_device(on_dev[it], None if use_rho else cost_dev, rho=rho if use_rho else None)
            torch.cuda.synchronize()
            # ---- the same iteration from the oracle's functions
            sel = orc.select_prefix_coverage(d["parent"], d["q"], rho, N) if use_rho else orc.select_prefix(d["parent"], d["q"], cost, N)
            keep, k = sel["keep"], sel["k_star"]
            assert int(loop.k_log[slot].item()) == k
            assert loop.keep[:k].tolist() == list(keep)
            par, x, tok, tn = sel["new_parent"], d["x"][keep], d["tok"][keep], d["target_next"][keep]
            outs, xin = [], x
            for l in range(n_layers):
                r = orc.verify_layer(cfg, Ws[l], np.array([0, k]), par, xin, [K[l]], [V[l]], np.array([L]))
                outs.append(r)
                xin = r["out"]
            path, bonus = orc.accept_path(par, tok, tn)
            plen = int(loop.plen_log[slot].item())
            assert plen == len(path) and loop.path[0, :plen].tolist() == list(path) and int(loop.bonus.item()) == bonus
            for l in range(n_layers):
                K[l], V[l] = orc.kv_commit(K[l], V[l], orc.handoff(outs[l]["k_new"], cfg.dtype),
                                           orc.handoff(outs[l]["v_new"], cfg.dtype), path)
            L += len(path)
            lens.append(len(path)); ks.append(k)
            assert int(loop.ctx_len[loop.cur].item()) == L and loop.ctx_len_host >= L
            tol = stack_tol(cfg.dtype, n_layers)
            assert rel_l2(harness.to_host(loop.out[:k]), outs[-1]["out"]) < tol, f"iteration {it}"
        assert max(lens) > 1 and min(ks) < N, (lens, ks)
        assert loop.resync() == L
        assert ev.evict_device_status(layers[0].ctx) == 0
    finally:
        ev.evict_dynamic_tokens(layers[0].ctx, None)
        layers[0].close()


def test_device_dispatched_iteration_is_one_graph():
    """The whole iteration (selection, compaction, layer stack, acceptance, commit) recorded once and replayed with
    refreshed inputs: every replay equals the same iteration made of direct calls (separate caches, same context
    bound, so the launches are identical), with eager work of the other loop between the replays."""
    cfg = synth.CONFIGS["mini_bf16"]
    n_layers, N, L0, cap, iters, seed = 2, 14, 37, 128, 4, 75
    Ws = [synth.layer_weights(cfg, synth.philox(seed, 1 + l)) for l in range(n_layers)]
    kv = [synth.kv_cache(cfg, L0, synth.philox(seed, 200 + l)) for l in range(n_layers)]
    drafts = [synth.draft_iteration(cfg, N, seed, it, 0.4, vocab=500) for it in range(iters)]
    cost_dev = torch.from_numpy((1.0 + 0.35 * np.arange(N + 1)).astype(np.float32)).to(DEV)
    layers = [harness.DeviceLayer(cfg, Ws[0], max_tokens=N, max_batch=1, max_ctx=cap)]
    for W in Ws[1:]:
        layers.append(harness.DeviceLayer(cfg, W, 0, 0, 0, ctx=layers[0].ctx))
    try:
        def make_loop():
            kc = [torch.zeros(1, cfg.Hkv, cap, cfg.D, dtype=torch.bfloat16, device=DEV) for _ in range(n_layers)]
            vc = [torch.zeros_like(k) for k in kc]
            for l in range(n_layers):
                kc[l][0, :, :L0] = harness.to_dev(kv[l][0], cfg.dtype)
                vc[l][0, :, :L0] = harness.to_dev(kv[l][1], cfg.dtype)
            lp = SpecLoop(cfg, layers[0].ctx, [l.weights for l in layers], kc, vc, cfg.Hkv * cap * cfg.D, cap * cfg.D, cap, N)
            lp.set_context_length(L0)
            return lp, kc, vc
        eager, kc_e, vc_e = make_loop()
        graphed, kc_g, vc_g = make_loop()
        on_dev = [to_device(cfg, d) for d in drafts]
        static = to_device(cfg, drafts[0])               # the graph's input buffers
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph = graphed.capture_on_device(static, cost_dev)
            side.synchronize()
            for it in range(iters):
                for name in ("parent", "q", "x", "tok", "target_next"):
                    getattr(static, name).copy_(getattr(on_dev[it], name))
                ev.evict_graph_launch(graph)
                side.synchronize()
                # the same iteration as direct calls on the other loop (eager work between the replays)
                eager.ctx_len_host = cap
                slot = eager.iteration_on_device(on_dev[it], cost_dev)
                side.synchronize()
                assert int(graphed.k_log[0].item()) == int(eager.k_log[slot].item())
                assert int(graphed.plen_log[0].item()) == int(eager.plen_log[slot].item())
                k = int(eager.k_log[slot].item())
                assert torch.equal(graphed.out[:k], eager.out[:k]) and torch.equal(graphed.path, eager.path)
                assert int(graphed.ctx_len[graphed.cur].item()) == int(eager.ctx_len[eager.cur].item())
            for l in range(n_layers):
                assert torch.equal(kc_g[l], kc_e[l]) and torch.equal(vc_g[l], vc_e[l])
            assert int(eager.ctx_len[eager.cur].item()) > L0 + iters   # some draft tokens were accepted
        ev.evict_graph_destroy(graph)
        assert ev.evict_device_status(layers[0].ctx) == 0
    finally:
        ev.evict_dynamic_tokens(layers[0].ctx, None)
        layers[0].close()
