"""GPU parity of the KV commit of accepted paths (bit-exact row copies at the right positions)
and of a second verification that reads the committed rows, against the CPU oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle import evict_oracle as orc

pytestmark = pytest.mark.gpu

ev = pytest.importorskip("paper_2605_00342_amd")
from paper_2605_00342_amd import harness  # noqa: E402

DEV = "cuda:0"
TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_l2(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-30))


class Cache:
    """KV cache with spare capacity, [B][Hkv][cap][D]."""

    def __init__(self, case, cap):
        cfg = case["cfg"]
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        B = len(case["ctx_len"])
        self.k = torch.zeros(B, cfg.Hkv, cap, cfg.D, dtype=tdt, device=DEV)
        self.v = torch.zeros_like(self.k)
        for b in range(B):
            L = int(case["ctx_len"][b])
            self.k[b, :, :L] = harness.to_dev(case["K"][b][:, :L], cfg.dtype)
            self.v[b, :, :L] = harness.to_dev(case["V"][b][:, :L], cfg.dtype)
        self.cap = cap
        self.seq_stride, self.head_stride = cfg.Hkv * cap * cfg.D, cap * cfg.D


def verify(layer, cfg, cache, tree_off, parent, ctx_len_dev, max_ctx, x):
    T = int(tree_off[-1])
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    out = torch.zeros(T, cfg.d, dtype=tdt, device=DEV)
    kn = torch.zeros(T, cfg.Hkv, cfg.D, dtype=tdt, device=DEV)
    vn = torch.zeros_like(kn)
    ev.evict_verify_layer(layer.ctx, layer.weights, harness.dev_i32(tree_off), harness.dev_i32(parent), len(tree_off) - 1, T,
                          cache.k, cache.v, cache.seq_stride, cache.head_stride, ctx_len_dev, max_ctx,
                          harness.to_dev(x, cfg.dtype), out, kn, vn, None)
    return out, kn, vn


@pytest.mark.parametrize("cfg_name,sizes,Ls", [("tiny", [8], [64]), ("mini_bf16", [24, 9, 40], [150, 31, 200])])
def test_commit_then_second_iteration(cfg_name, sizes, Ls):
    B = len(sizes)
    case = synth.make_case(cfg_name, n=sizes[0], L=Ls[0], seed=17, batch=B, L_list=Ls) if B > 1 else \
        synth.make_case(cfg_name, n=sizes[0], L=Ls[0], seed=17)
    cfg = case["cfg"]
    tree_off, parent = case["tree_off"], case["parent"]
    sizes = [int(tree_off[b + 1] - tree_off[b]) for b in range(B)]
    cap = max(Ls) + 64
    layer = harness.DeviceLayer(cfg, case["W"], max_tokens=int(tree_off[-1]), max_batch=B, max_ctx=cap)
    try:
        cache = Cache(case, cap)
        ctx_len = harness.dev_i32(case["ctx_len"])
        out1, kn, vn = verify(layer, cfg, cache, tree_off, parent, ctx_len, max(Ls), case["x"])
        ref1 = orc.verify_layer(cfg, case["W"], tree_off, parent, case["x"], case["K"], case["V"], case["ctx_len"])
        assert rel_l2(harness.to_host(out1), ref1["out"]) < TOL[cfg.dtype]

        # accepted paths: the root path of the deepest node of each tree
        stride = max(sizes)
        path = np.full((B, stride), -1, np.int32)
        plen = np.zeros(B, np.int32)
        paths = []
        for b in range(B):
            par = parent[tree_off[b]:tree_off[b + 1]]
            depth = np.zeros(len(par), int)
            for i in range(1, len(par)):
                depth[i] = depth[par[i]] + 1
            node, p = int(np.argmax(depth)), []
            while node >= 0:
                p.append(node)
                node = int(par[node])
            p = p[::-1]
            paths.append(p)
            path[b, :len(p)] = p
            plen[b] = len(p)
        k_before, v_before = cache.k.clone(), cache.v.clone()
        ctx_len2 = torch.zeros(B, dtype=torch.int32, device=DEV)
        ev.evict_kv_commit(layer.ctx, ev.EVICT_BF16 if cfg.dtype == "bf16" else ev.EVICT_F32, cfg.Hkv, cfg.D, kn, vn,
                           harness.dev_i32(tree_off), harness.dev_i32(path), stride, harness.dev_i32(plen), cache.k, cache.v,
                           cache.seq_stride, cache.head_stride, ctx_len, cap, ctx_len2, B)
        torch.cuda.synchronize()
        assert ev.evict_device_status(layer.ctx) == 0
        # bit-exact: committed rows are the draft rows; everything else is untouched
        new_len = ctx_len2.cpu().numpy()
        want_k, want_v = k_before.clone(), v_before.clone()
        for b in range(B):
            L = int(case["ctx_len"][b])
            assert new_len[b] == L + len(paths[b])
            for j, node in enumerate(paths[b]):
                want_k[b, :, L + j] = kn[tree_off[b] + node]
                want_v[b, :, L + j] = vn[tree_off[b] + node]
        assert torch.equal(cache.k, want_k) and torch.equal(cache.v, want_v)

        # second iteration: new trees on the extended caches, GPU vs oracle (the oracle commits its own rows)
        K2, V2 = [], []
        for b in range(B):
            lo, hi = tree_off[b], tree_off[b + 1]
            k2, v2 = orc.kv_commit(case["K"][b], case["V"][b], orc.handoff(ref1["k_new"][lo:hi], cfg.dtype),
                                   orc.handoff(ref1["v_new"][lo:hi], cfg.dtype), paths[b])
            K2.append(k2); V2.append(v2)
        g = synth.philox(17, 88)
        pars2 = [synth.tree_bfs_random(n, g) for n in sizes]
        off2, par2 = synth.concat_trees(pars2)
        x2 = np.concatenate([synth.hidden_states(p, cfg.d, 0.5, g, cfg.dtype) for p in pars2])
        out2, _, _ = verify(layer, cfg, cache, off2, par2, ctx_len2, int(new_len.max()), x2)
        ref2 = orc.verify_layer(cfg, case["W"], off2, par2, x2, K2, V2, new_len)
        assert rel_l2(harness.to_host(out2), ref2["out"]) < TOL[cfg.dtype]
    finally:
        layer.close()


def test_commit_capacity_and_bad_entries():
    cfg = synth.CONFIGS["tiny"]
    case = synth.make_case("tiny", n=8, L=60, seed=5, tree="chain")
    layer = harness.DeviceLayer(cfg, case["W"], max_tokens=8, max_batch=1, max_ctx=64)
    try:
        cache = Cache(case, 64)  # 4 free rows
        kn = torch.randn(8, cfg.Hkv, cfg.D, device=DEV)
        vn = torch.randn(8, cfg.Hkv, cfg.D, device=DEV)
        path = np.arange(8, dtype=np.int32)[None]
        out_len = torch.zeros(1, dtype=torch.int32, device=DEV)
        args = (layer.ctx, ev.EVICT_F32, cfg.Hkv, cfg.D, kn, vn, harness.dev_i32(case["tree_off"]), harness.dev_i32(path), 8,
                harness.dev_i32(np.array([6], np.int32)), cache.k, cache.v, cache.seq_stride, cache.head_stride)
        ctx_len = harness.dev_i32(case["ctx_len"])
        ev.evict_kv_commit(*args, ctx_len, 64, out_len, 1)
        torch.cuda.synchronize()
        assert int(out_len[0]) == 64                       # clamped to the capacity
        assert torch.equal(cache.k[0, :, 60:64], kn[:4].transpose(0, 1))
        assert ev.evict_device_status(layer.ctx) != 0      # and reported
        with pytest.raises(ev.EvictError):                 # the new length must not alias the old one
            ev.evict_kv_commit(*args, ctx_len, 64, ctx_len, 1)
        # a path that evict_accept_path had to truncate (path_len > path_stride): the rows that are there are
        # committed, the length advances by that many, and the call is flagged
        layer2 = harness.DeviceLayer(cfg, case["W"], max_tokens=8, max_batch=1, max_ctx=64)
        cache2 = Cache(case, 64)
        short = harness.dev_i32(np.array([[0, 1, 2]], np.int32))
        ctx50 = harness.dev_i32(np.array([50], np.int32))
        ev.evict_kv_commit(layer2.ctx, ev.EVICT_F32, cfg.Hkv, cfg.D, kn, vn, harness.dev_i32(case["tree_off"]), short, 3,
                           harness.dev_i32(np.array([5], np.int32)), cache2.k, cache2.v, cache2.seq_stride, cache2.head_stride,
                           ctx50, 64, out_len, 1)
        torch.cuda.synchronize()
        assert int(out_len[0]) == 53
        assert torch.equal(cache2.k[0, :, 50:53], kn[:3].transpose(0, 1))
        assert ev.evict_device_status(layer2.ctx) == 32
        layer2.close()
        with pytest.raises(ev.EvictError):                 # strides too small for the capacity
            ev.evict_kv_commit(*args[:12], cache.seq_stride, 10, ctx_len, 64, out_len, 1)
    finally:
        layer.close()
