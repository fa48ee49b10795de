"""Paged KV caches (block table + page pools) through the C ABI: the paged stack must equal the
contiguous one bit for bit (same kernels, only the key addresses differ) and the CPU oracle
within tolerance; the paged commit must place the accepted rows exactly; a second iteration reads
them back; bad page ids are flagged and never followed."""
import numpy as np
import pytest
import torch

import synth
from oracle import evict_oracle as orc

pytestmark = pytest.mark.gpu

ev = pytest.importorskip("paper_2605_00342_amd")
from paper_2605_00342_amd import harness  # noqa: E402

DEV = "cuda:0"
from tolerances import TOL, stack_tol  # noqa: E402,F401
NL = 2


def rel_l2(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-30))


def tdt(cfg):
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


def build(cfg_name, n, Ls, P, seed, extra):
    """Case, per-layer weights and caches, and their paged form (one table for all layers)."""
    B = len(Ls)
    case = synth.make_case(cfg_name, n=n, L=Ls[0], seed=seed, batch=B, L_list=Ls)
    cfg = case["cfg"]
    Ws = [case["W"]] + [synth.layer_weights(cfg, synth.philox(seed, 1000 + l)) for l in range(1, NL)]
    Ks, Vs = [case["K"]], [case["V"]]
    for l in range(1, NL):
        kv = [synth.kv_cache(cfg, int(Lb), synth.philox(seed, 2000 + 10 * l + b)) for b, Lb in enumerate(Ls)]
        Ks.append([k for k, _ in kv]); Vs.append([v for _, v in kv])
    pools, table, n_pages = [], None, 0
    for l in range(NL):
        pk, pv, tb, n_pages = synth.to_pages(Ks[l], Vs[l], P, [L + extra for L in Ls], synth.philox(seed, 77))
        assert table is None or np.array_equal(table, tb)
        table = tb
        pools.append((pk, pv))
    return case, cfg, Ws, Ks, Vs, pools, table, n_pages


class Dev:
    """Device side of a built case: context + layers, contiguous caches and page pools."""

    def __init__(self, case, cfg, Ws, Ks, Vs, pools, table, n_pages, P, cap):
        self.cfg, self.P, self.n_pages, self.cap = cfg, P, n_pages, cap
        self.B, self.T = len(case["ctx_len"]), int(case["tree_off"][-1])
        self.layers = [harness.DeviceLayer(cfg, Ws[0], self.T, self.B, cap)]
        self.ctx = self.layers[0].ctx
        self.layers += [harness.DeviceLayer(cfg, W, 0, 0, 0, ctx=self.ctx) for W in Ws[1:]]
        self.weights = [l.weights for l in self.layers]
        self.kc, self.vc = [], []
        for l in range(NL):
            k = torch.zeros(self.B, cfg.Hkv, cap, cfg.D, dtype=tdt(cfg), device=DEV)
            v = torch.zeros_like(k)
            for b in range(self.B):
                L = int(case["ctx_len"][b])
                k[b, :, :L] = harness.to_dev(Ks[l][b], cfg.dtype)
                v[b, :, :L] = harness.to_dev(Vs[l][b], cfg.dtype)
            self.kc.append(k); self.vc.append(v)
        self.pk = [harness.to_dev(p[0], cfg.dtype) for p in pools]
        self.pv = [harness.to_dev(p[1], cfg.dtype) for p in pools]
        self.table = harness.dev_i32(table)
        self.table_stride = table.shape[1]
        self.page_stride, self.head_stride = cfg.Hkv * P * cfg.D, P * cfg.D

    def bufs(self, T):
        cfg = self.cfg
        out = torch.zeros(T, cfg.d, dtype=tdt(cfg), device=DEV)
        kn = [torch.zeros(T, cfg.Hkv, cfg.D, dtype=tdt(cfg), device=DEV) for _ in range(NL)]
        vn = [torch.zeros_like(k) for k in kn]
        return out, kn, vn

    def run_contiguous(self, tree_off, parent, ctx_len, max_ctx, x):
        T = int(tree_off[-1])
        out, kn, vn = self.bufs(T)
        ev.evict_verify_stack(self.ctx, self.weights, harness.dev_i32(tree_off), harness.dev_i32(parent), self.B, T, self.kc,
                              self.vc, self.cfg.Hkv * self.cap * self.cfg.D, self.cap * self.cfg.D, ctx_len, max_ctx,
                              harness.to_dev(x, self.cfg.dtype), out, kn, vn)
        return out, kn, vn

    def run_paged(self, tree_off, parent, ctx_len, max_ctx, x, table=None):
        T = int(tree_off[-1])
        out, kn, vn = self.bufs(T)
        ev.evict_verify_stack_paged(self.ctx, self.weights, harness.dev_i32(tree_off), harness.dev_i32(parent), self.B, T, self.pk,
                                    self.pv, self.page_stride, self.head_stride, self.table if table is None else table,
                                    self.table_stride, self.P, self.n_pages, ctx_len, max_ctx,
                                    harness.to_dev(x, self.cfg.dtype), out, kn, vn)
        return out, kn, vn

    def close(self):
        for l in self.layers[1:]:
            l.close()
        self.layers[0].close()


def oracle_stack(cfg, Ws, Ks, Vs, tree_off, parent, x, ctx_len):
    outs = []
    for l in range(NL):
        r = orc.verify_layer(cfg, Ws[l], tree_off, parent, x, Ks[l], Vs[l], ctx_len)
        outs.append(r)
        x = r["out"]
    return outs


def deepest_paths(tree_off, parent):
    paths = []
    for b in range(len(tree_off) - 1):
        par = parent[tree_off[b]:tree_off[b + 1]]
        depth = np.zeros(len(par), int)
        for i in range(1, len(par)):
            depth[i] = depth[par[i]] + 1
        node, p = int(np.argmax(depth)), []
        while node >= 0:
            p.append(node)
            node = int(par[node])
        paths.append(p[::-1])
    return paths


@pytest.mark.parametrize("cfg_name,n,Ls,P", [
    ("tiny", 8, [64], 16), ("tiny", 9, [37, 0, 5], 4), ("mini_bf16", 24, [150, 31, 300], 16),
    ("mini_bf16", 40, [700], 64), ("mini_bf16", 20, [130], 1), ("mini_bf16", 33, [260, 129], 256),
    ("mini_sigmoid", 16, [200, 90], 32), ("mini_bf16", 12, [20000, 777], 16),
])
def test_paged_stack_commit_and_second_iteration(cfg_name, n, Ls, P):
    extra = 40
    case, cfg, Ws, Ks, Vs, pools, table, n_pages = build(cfg_name, n, Ls, P, 23, extra)
    B, tree_off, parent = len(Ls), case["tree_off"], case["parent"]
    cap = max(Ls) + extra
    d = Dev(case, cfg, Ws, Ks, Vs, pools, table, n_pages, P, cap)
    try:
        ctx_len = harness.dev_i32(case["ctx_len"])
        out_c, kn_c, vn_c = d.run_contiguous(tree_off, parent, ctx_len, max(Ls), case["x"])
        out_p, kn_p, vn_p = d.run_paged(tree_off, parent, ctx_len, max(Ls), case["x"])
        torch.cuda.synchronize()
        assert ev.evict_device_status(d.ctx) == 0          # in particular: no table entry past a sequence's pages was read
        assert torch.equal(out_p, out_c)
        for l in range(NL):
            assert torch.equal(kn_p[l], kn_c[l]) and torch.equal(vn_p[l], vn_c[l])
        # the oracle reads the same pools through the table
        Kv = [[orc.paged_view(pools[l][0], table[b], Ls[b], P) for b in range(B)] for l in range(NL)]
        Vv = [[orc.paged_view(pools[l][1], table[b], Ls[b], P) for b in range(B)] for l in range(NL)]
        ref = oracle_stack(cfg, Ws, Kv, Vv, tree_off, parent, case["x"], case["ctx_len"])
        assert rel_l2(harness.to_host(out_p), ref[-1]["out"]) < stack_tol(cfg.dtype, NL)

        # ---- commit of one accepted path per sequence into the pages
        paths = deepest_paths(tree_off, parent)
        stride = n
        path = np.full((B, stride), -1, np.int32)
        plen = np.array([len(p) for p in paths], np.int32)
        for b, p in enumerate(paths):
            path[b, :len(p)] = p
        want = []
        for l in range(NL):
            wk, wv = harness.to_host(d.pk[l]).copy(), harness.to_host(d.pv[l]).copy()
            knh, vnh = harness.to_host(kn_p[l]), harness.to_host(vn_p[l])
            for b in range(B):
                lo, hi = tree_off[b], tree_off[b + 1]
                orc.kv_commit_paged(wk, wv, table[b], Ls[b], knh[lo:hi], vnh[lo:hi], paths[b], P)
            want.append((wk, wv))
        ctx_len2 = torch.zeros(B, dtype=torch.int32, device=DEV)
        ev.evict_kv_commit_stack_paged(d.ctx, ev.EVICT_BF16 if cfg.dtype == "bf16" else ev.EVICT_F32, cfg.Hkv, cfg.D, kn_p, vn_p,
                                       harness.dev_i32(tree_off), harness.dev_i32(path), stride, harness.dev_i32(plen), d.pk, d.pv,
                                       d.page_stride, d.head_stride, d.table, d.table_stride, P, n_pages, ctx_len, cap,
                                       ctx_len2, B)
        torch.cuda.synchronize()
        assert ev.evict_device_status(d.ctx) == 0
        new_len = ctx_len2.cpu().numpy()
        assert np.array_equal(new_len, np.asarray(Ls) + plen)
        for l in range(NL):
            assert np.array_equal(harness.to_host(d.pk[l]), want[l][0]) and np.array_equal(harness.to_host(d.pv[l]), want[l][1])

        # ---- second iteration on the extended paged caches; the oracle commits its own rows
        K2 = [[None] * B for _ in range(NL)]
        V2 = [[None] * B for _ in range(NL)]
        for l in range(NL):
            for b in range(B):
                lo, hi = tree_off[b], tree_off[b + 1]
                K2[l][b], V2[l][b] = orc.kv_commit(Kv[l][b], Vv[l][b], orc.handoff(ref[l]["k_new"][lo:hi], cfg.dtype),
                                                   orc.handoff(ref[l]["v_new"][lo:hi], cfg.dtype), paths[b])
        g = synth.philox(23, 88)
        pars2 = [synth.tree_bfs_random(n, g) for _ in range(B)]
        off2, par2 = synth.concat_trees(pars2)
        x2 = np.concatenate([synth.hidden_states(p, cfg.d, 0.5, g, cfg.dtype) for p in pars2])
        out2, _, _ = d.run_paged(off2, par2, ctx_len2, int(new_len.max()), x2)
        ref2 = oracle_stack(cfg, Ws, K2, V2, off2, par2, x2, new_len)
        assert rel_l2(harness.to_host(out2), ref2[-1]["out"]) < stack_tol(cfg.dtype, NL)
        assert ev.evict_device_status(d.ctx) == 0
    finally:
        d.close()


def test_bad_page_ids_are_flagged_and_never_followed():
    P, Ls, n = 16, [50], 8
    case, cfg, Ws, Ks, Vs, pools, table, n_pages = build("tiny", n, Ls, P, 29, 20)
    d = Dev(case, cfg, Ws, Ks, Vs, pools, table, n_pages, P, Ls[0] + 20)
    try:
        ctx_len = harness.dev_i32(case["ctx_len"])
        bad = table.copy()
        bad[0, 1] = n_pages + 1000           # positions 16..31: far outside the pool
        out, kn, vn = d.run_paged(case["tree_off"], case["parent"], ctx_len, Ls[0], case["x"], table=harness.dev_i32(bad))
        torch.cuda.synchronize()
        assert ev.evict_device_status(d.ctx) & 16
        assert bool(torch.isfinite(out.float()).all())
    finally:
        d.close()
    # a commit into a bad page writes nothing there and flags it (fresh context: the status word is sticky)
    d = Dev(case, cfg, Ws, Ks, Vs, pools, table, n_pages, P, Ls[0] + 20)
    try:
        ctx_len = harness.dev_i32(case["ctx_len"])
        out, kn, vn = d.run_paged(case["tree_off"], case["parent"], ctx_len, Ls[0], case["x"])
        torch.cuda.synchronize()
        assert ev.evict_device_status(d.ctx) == 0
        bad2 = table.copy()
        bad2[0, 3] = -7                      # positions 48..63: the commit starts at 50
        before_k = [p.clone() for p in d.pk]
        path = np.array([[0, 1, 2, 3, 4, 5, 6, 7]], np.int32)
        ctx_len2 = torch.zeros(1, dtype=torch.int32, device=DEV)
        ev.evict_kv_commit_stack_paged(d.ctx, ev.EVICT_F32, cfg.Hkv, cfg.D, kn, vn, harness.dev_i32(np.array([0, n])),
                                       harness.dev_i32(path), n, harness.dev_i32(np.array([n])), d.pk, d.pv, d.page_stride,
                                       d.head_stride, harness.dev_i32(bad2), d.table_stride, P, n_pages, ctx_len, Ls[0] + 20,
                                       ctx_len2, 1)
        torch.cuda.synchronize()
        assert ev.evict_device_status(d.ctx) & 16
        for l in range(NL):
            assert torch.equal(d.pk[l], before_k[l])
    finally:
        d.close()


def test_paged_argument_errors():
    P, Ls, n = 16, [40], 8
    case, cfg, Ws, Ks, Vs, pools, table, n_pages = build("tiny", n, Ls, P, 31, 8)
    d = Dev(case, cfg, Ws, Ks, Vs, pools, table, n_pages, P, 48)
    try:
        ctx_len = harness.dev_i32(case["ctx_len"])
        T = n
        out, kn, vn = d.bufs(T)
        off, par, x = harness.dev_i32(case["tree_off"]), harness.dev_i32(case["parent"]), harness.to_dev(case["x"], cfg.dtype)

        def call(page_size=P, table_stride=d.table_stride, n_pages_=n_pages, head_stride=d.head_stride, page_stride=d.page_stride):
            ev.evict_verify_stack_paged(d.ctx, d.weights, off, par, 1, T, d.pk, d.pv, page_stride, head_stride, d.table, table_stride,
                                        page_size, n_pages_, ctx_len, Ls[0], x, out, kn, vn)
        for kw in (dict(page_size=12), dict(page_size=0), dict(table_stride=2), dict(n_pages_=0), dict(head_stride=P * cfg.D - 8),
                   dict(page_stride=d.page_stride - 8)):
            with pytest.raises(ev.EvictError):
                call(**kw)
        call()                                               # and the context still works, unpaged state restored
        out_c, _, _ = d.run_contiguous(case["tree_off"], case["parent"], ctx_len, Ls[0], case["x"])
        torch.cuda.synchronize()
        assert torch.equal(out, out_c)
    finally:
        d.close()
