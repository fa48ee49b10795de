"""HIP-graph capture of the verification step (one pre-built graph per verification length,
Sec. 3.3): every replay must reproduce the directly launched calls bit for bit, also after the
inputs were refreshed in place and with the program's own eager work between replays; the
directly launched calls are themselves checked against the CPU oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle import evict_oracle as orc

pytestmark = pytest.mark.gpu

ev = pytest.importorskip("paper_2605_00342_amd")
from paper_2605_00342_amd import harness  # noqa: E402

DEV = "cuda:0"


def rel_l2(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-30))


class StepBuffers:
    """select_prefix + verify_layer + accept_path of one tree, with every output in its own buffer."""

    def __init__(self, case, dc, layer, vocab=1000):
        i32, f32 = torch.int32, torch.float32
        N = dc.T
        self.case, self.dc, self.layer, self.N = case, dc, layer, N
        cfg = case["cfg"]
        self.q = torch.from_numpy(case["q"]).to(DEV)
        self.cost = torch.from_numpy(synth.cost_linear_in_union(N, cfg.E, cfg.k)).to(DEV)
        self.k_star = torch.zeros(1, dtype=i32, device=DEV)
        self.keep = torch.zeros(N, dtype=i32, device=DEV)
        self.new_parent = torch.zeros(N, dtype=i32, device=DEV)
        self.new_off = torch.zeros(2, dtype=i32, device=DEV)
        self.est = torch.zeros(1, dtype=f32, device=DEV)
        g = synth.philox(77, 900)
        self.target_next_np = g.integers(0, vocab, N).astype(np.int32)
        self.draft_tok_np = synth.plant_draft_tokens(case["parent"], self.target_next_np, vocab, g)
        self.tn, self.dt = harness.dev_i32(self.target_next_np), harness.dev_i32(self.draft_tok_np)
        self.path = torch.zeros(1, N, dtype=i32, device=DEV)
        self.path_len = torch.zeros(1, dtype=i32, device=DEV)
        self.bonus = torch.zeros(1, dtype=i32, device=DEV)

    def step(self):
        dc, N = self.dc, self.N
        ev.evict_select_prefix(None, dc.tree_off, dc.parent, self.q, 1, N, self.cost, N, self.k_star, self.keep,
                               self.new_parent, self.new_off, self.est)
        dc.run(self.layer)
        ev.evict_accept_path(None, dc.tree_off, dc.parent, self.dt, self.tn, 1, self.path, N, self.path_len, self.bonus)

    def outputs(self):
        dc = self.dc
        return [t.clone() for t in (dc.out, dc.k_new, dc.v_new, self.k_star, self.keep, self.new_parent, self.est,
                                    self.path, self.path_len, self.bonus, dc.a["topk_idx"], dc.a["union_ids"])]

    def clear(self):
        dc = self.dc
        for t in (dc.out, dc.k_new, dc.v_new, self.k_star, self.keep, self.new_parent, self.est, self.path,
                  self.path_len, self.bonus, dc.a["topk_idx"], dc.a["union_ids"]):
            t.zero_()


@pytest.mark.parametrize("cfg_name,n,L", [("tiny", 8, 64), ("mini_bf16", 40, 300)])
def test_graph_replays_match_direct_calls(cfg_name, n, L):
    case = synth.make_case(cfg_name, n=n, L=L, seed=31)
    cfg = case["cfg"]
    layer = harness.DeviceLayer(cfg, case["W"], max_tokens=n, max_batch=1, max_ctx=L)
    dc = harness.DeviceCase(case, with_aux=True)
    sb = StepBuffers(case, dc, layer)
    side = torch.cuda.Stream()
    graph = None
    try:
        with torch.cuda.stream(side):
            # direct calls first: reference outputs, checked against the oracle
            sb.step()
            side.synchronize()
            ref = sb.outputs()
            want = orc.verify_layer(cfg, case["W"], case["tree_off"], case["parent"], case["x"], case["K"], case["V"],
                                    case["ctx_len"])
            tol = 1e-4 if cfg.dtype == "f32" else 2e-2
            assert rel_l2(harness.to_host(dc.out), want["out"]) < tol
            path, bonus = orc.accept_path(case["parent"], sb.draft_tok_np, sb.target_next_np)
            assert harness.to_host(sb.path_len)[0] == len(path) and harness.to_host(sb.bonus)[0] == bonus

            ev.evict_graph_begin(layer.ctx)
            sb.step()
            graph = ev.evict_graph_end(layer.ctx)

            x0 = dc.x.clone()
            q0 = sb.q.clone()
            for rep in range(4):
                if rep == 2:
                    # inputs refreshed in place: other hidden states and draft probabilities
                    g = torch.Generator(device="cpu").manual_seed(5)
                    dc.x.copy_((x0.float().cpu() + 0.25 * torch.randn(x0.shape, generator=g)).to(x0.dtype))
                    sb.q.copy_(torch.clamp(q0 * 0.5 + 0.2, 0.05, 1.0))
                    sb.clear()
                    sb.step()  # eager work of the program's own between replays
                    side.synchronize()
                    ref = sb.outputs()
                sb.clear()
                ev.evict_graph_launch(graph)
                side.synchronize()
                got = sb.outputs()
                for a, b in zip(got, ref):
                    assert torch.equal(a, b), f"replay {rep} differs from the direct calls"
    finally:
        if graph is not None:
            ev.evict_graph_destroy(graph)
        layer.close()


def test_graph_error_paths():
    case = synth.make_case("tiny", n=8, L=64, seed=3)
    layer = harness.DeviceLayer(case["cfg"], case["W"], max_tokens=8, max_batch=1, max_ctx=64)
    try:
        with pytest.raises(ev.EvictError):  # the null stream cannot be captured
            ev.evict_graph_begin(layer.ctx)
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            with pytest.raises(ev.EvictError):  # no capture open
                ev.evict_graph_end(layer.ctx)
            ev.evict_stage_timing(layer.ctx, True)
            with pytest.raises(ev.EvictError):  # stage timing records events
                ev.evict_graph_begin(layer.ctx)
            ev.evict_stage_timing(layer.ctx, False)
            # (buffers are allocated before the capture opens: an allocation would invalidate it)
            keep = torch.arange(8, dtype=torch.int32, device=DEV)
            off = torch.tensor([0, 8], dtype=torch.int32, device=DEV)
            src = torch.ones(8, 4, device=DEV)
            dst = torch.zeros(8, 4, device=DEV)
            side.synchronize()
            ev.evict_graph_begin(layer.ctx)
            with pytest.raises(ev.EvictError):  # already open
                ev.evict_graph_begin(layer.ctx)
            ev.evict_gather_rows(src, dst, 16, off, off, keep, 1, 8)
            g = ev.evict_graph_end(layer.ctx)
            side.synchronize()
            assert float(dst.sum()) == 0.0  # recorded, not run
            ev.evict_graph_launch(g)
            side.synchronize()
            assert float(dst.sum()) == 32.0
            side.synchronize()
            ev.evict_graph_destroy(g)
    finally:
        layer.close()


def test_one_graph_per_verification_length_dispatched_by_the_selected_length():
    """Sec. 3.3: the verification of every length k is captured once; at run time the selection runs, its k* is
    read back and the graph of that length is replayed on the compacted tree. Every replay must equal the
    direct calls for the same k* bit for bit."""
    N, L = 12, 50
    case = synth.make_case("mini_bf16", n=N, L=L, seed=41)
    cfg = case["cfg"]
    layer = harness.DeviceLayer(cfg, case["W"], max_tokens=N, max_batch=1, max_ctx=L)
    dc = harness.DeviceCase(case, with_aux=False)
    i32, f32 = torch.int32, torch.float32
    tdt = torch.bfloat16
    side = torch.cuda.Stream()
    graphs = {}
    try:
        with torch.cuda.stream(side):
            q = torch.from_numpy(case["q"]).to(DEV)
            cost = torch.zeros(N + 1, dtype=f32, device=DEV)
            k_star = torch.zeros(1, dtype=i32, device=DEV); keep = torch.zeros(N, dtype=i32, device=DEV)
            new_parent = torch.zeros(N, dtype=i32, device=DEV); new_off = torch.zeros(2, dtype=i32, device=DEV)
            est = torch.zeros(1, dtype=f32, device=DEV)
            xg = torch.zeros(N, cfg.d, dtype=tdt, device=DEV)
            out = torch.zeros(N, cfg.d, dtype=tdt, device=DEV)
            kn = torch.zeros(N, cfg.Hkv, cfg.D, dtype=tdt, device=DEV); vn = torch.zeros_like(kn)

            def verify(k):
                ev.evict_gather_rows(dc.x, xg, cfg.d * 2, dc.tree_off, new_off, keep, 1, N)
                ev.evict_verify_layer(layer.ctx, layer.weights, new_off, new_parent, 1, k, dc.k_cache, dc.v_cache, dc.seq_stride,
                                      dc.head_stride, dc.ctx_len, L, xg, out, kn, vn, None)
            side.synchronize()
            for k in range(1, N + 1):
                ev.evict_graph_begin(layer.ctx)
                verify(k)
                graphs[k] = ev.evict_graph_end(layer.ctx)
            seen = set()
            for slope in (0.0, 0.02, 0.08, 0.3, 2.0):
                cost_np = (1.0 + slope * np.arange(N + 1)).astype(np.float32)
                cost.copy_(torch.from_numpy(cost_np))
                ev.evict_select_prefix(None, dc.tree_off, dc.parent, q, 1, N, cost, N, k_star, keep, new_parent, new_off, est)
                k = int(k_star.item())                      # the one read-back that picks the graph
                assert k == orc.select_prefix(case["parent"], case["q"], cost_np, N)["k_star"]
                seen.add(k)
                out.zero_(); kn.zero_()
                verify(k)
                side.synchronize()
                want_out, want_kn = out[:k].clone(), kn[:k].clone()
                out.zero_(); kn.zero_()
                ev.evict_graph_launch(graphs[k])
                side.synchronize()
                assert torch.equal(out[:k], want_out) and torch.equal(kn[:k], want_kn), f"k* = {k}"
            assert len(seen) >= 3, seen
    finally:
        for g in graphs.values():
            ev.evict_graph_destroy(g)
        layer.close()
