"""Host-side plumbing around the C ABI: upload numpy inputs as torch device tensors, pack
weights once, allocate outputs, call the library, download results. No arithmetic of the
method happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as ev


def storage_code(dtype: str) -> int:
    return ev.EVICT_BF16 if dtype == "bf16" else ev.EVICT_F32


def model_desc(cfg, vocab: int = 0) -> ev.ModelDesc:
    return ev.ModelDesc(storage_code(cfg.dtype), cfg.d, cfg.Hq, cfg.Hkv, cfg.D, cfg.E, cfg.k, cfg.F, cfg.n_shared,
                        cfg.eps, cfg.theta, vocab, 1 if getattr(cfg, "router_norm", "softmax") == "sigmoid" else 0)


def to_dev(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Upload values in the storage dtype. bf16 values must already be bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    t = torch.from_numpy(a).to(device)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def dev_i32(a, device="cuda:0") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)


class DeviceLayer:
    """Context + packed weights of one layer on the GPU."""

    def __init__(self, cfg, W, max_tokens, max_batch, max_ctx, device="cuda:0", vocab=0, ctx=None):
        self.cfg, self.device = cfg, device
        self.desc = model_desc(cfg, vocab)
        self.owns_ctx = ctx is None
        self.ctx = ev.evict_create(self.desc, max_tokens, max_batch, max_ctx) if ctx is None else ctx
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        eb = 2 if cfg.dtype == "bf16" else 4
        code = storage_code(cfg.dtype)

        def up(name):
            # (a tensor already on the device in the storage dtype is used as it is: stacks whose layers are
            # windows of one uploaded array pack straight from views of it)
            if isinstance(W[name], torch.Tensor):
                return W[name].contiguous()
            return to_dev(W[name], cfg.dtype, device)

        def empty(nbytes):
            return torch.empty(nbytes // eb, dtype=tdt, device=device)

        self.g_attn, self.g_moe = up("g_attn"), up("g_moe")
        wg_raw = up("wg")
        self.wg = empty(cfg.E * cfg.d * eb)
        ev.evict_pack_dense(code, wg_raw, cfg.E, cfg.d, self.wg)
        wq, wk, wv, wo = up("wq"), up("wk"), up("wv"), up("wo")
        self.wqkv = empty((cfg.Hq + 2 * cfg.Hkv) * cfg.D * cfg.d * eb)
        ev.evict_pack_qkv(self.desc, wq, wk, wv, self.wqkv)
        self.wo = empty(cfg.d * cfg.Hq * cfg.D * eb)
        ev.evict_pack_dense(code, wo, cfg.d, cfg.Hq * cfg.D, self.wo)
        self.w_gateup = empty(cfg.E * 2 * cfg.F * cfg.d * eb)
        self.w_down = empty(cfg.E * cfg.F * cfg.d * eb)
        g, u, dn = up("w_gate"), up("w_up"), up("w_down")
        ev.evict_pack_experts(self.desc, cfg.E, g, u, dn, self.w_gateup, self.w_down)
        self.ws_gateup = self.ws_down = None
        if cfg.n_shared:
            self.ws_gateup = empty(cfg.n_shared * 2 * cfg.F * cfg.d * eb)
            self.ws_down = empty(cfg.n_shared * cfg.F * cfg.d * eb)
            g2, u2, d2 = up("ws_gate"), up("ws_up"), up("ws_down")
            ev.evict_pack_experts(self.desc, cfg.n_shared, g2, u2, d2, self.ws_gateup, self.ws_down)
        torch.cuda.synchronize()
        del wq, wk, wv, wo, g, u, dn
        self.weights = ev.LayerWeights(self.g_attn.data_ptr(), self.g_moe.data_ptr(), self.wqkv.data_ptr(),
                                       self.wo.data_ptr(), self.wg.data_ptr(), self.w_gateup.data_ptr(),
                                       self.w_down.data_ptr(),
                                       self.ws_gateup.data_ptr() if cfg.n_shared else None,
                                       self.ws_down.data_ptr() if cfg.n_shared else None)

    def close(self):
        if self.ctx and self.owns_ctx:
            ev.evict_destroy(self.ctx)
        self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class DeviceCase:
    """Inputs of one verification call on the GPU plus output buffers."""

    def __init__(self, case, device="cuda:0", with_aux=True):
        cfg = case["cfg"]
        self.cfg = cfg
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.B = len(case["ctx_len"])
        self.T = int(case["tree_off"][-1])
        self.tree_off = dev_i32(case["tree_off"], device)
        self.parent = dev_i32(case["parent"], device)
        self.ctx_len = dev_i32(case["ctx_len"], device)
        self.max_ctx = int(max(case["ctx_len"]))
        cap = max(self.max_ctx, 1)
        kc = torch.zeros(self.B, cfg.Hkv, cap, cfg.D, dtype=tdt, device=device)
        vc = torch.zeros_like(kc)
        for b in range(self.B):
            L = int(case["ctx_len"][b])
            kc[b, :, :L] = to_dev(case["K"][b][:, :L], cfg.dtype, device)
            vc[b, :, :L] = to_dev(case["V"][b][:, :L], cfg.dtype, device)
        self.k_cache, self.v_cache = kc, vc
        self.seq_stride, self.head_stride = cfg.Hkv * cap * cfg.D, cap * cfg.D
        self.x = to_dev(case["x"], cfg.dtype, device)
        T = self.T
        self.out = torch.zeros(T, cfg.d, dtype=tdt, device=device)
        self.k_new = torch.zeros(T, cfg.Hkv, cfg.D, dtype=tdt, device=device)
        self.v_new = torch.zeros_like(self.k_new)
        self.aux = None
        if with_aux:
            i32, f32 = torch.int32, torch.float32
            self.a = {
                "h": torch.zeros(T, cfg.d, dtype=tdt, device=device),
                "h_norm": torch.zeros(T, cfg.d, dtype=tdt, device=device),
                "router_logits": torch.zeros(T, cfg.E, dtype=f32, device=device),
                "topk_idx": torch.zeros(T, cfg.k, dtype=i32, device=device),
                "topk_w": torch.zeros(T, cfg.k, dtype=f32, device=device),
                "union_ids": torch.zeros(cfg.E, dtype=i32, device=device),
                "union_count": torch.zeros(1, dtype=i32, device=device),
                "hist": torch.zeros(cfg.E, dtype=i32, device=device),
                "q": torch.zeros(T, cfg.Hq, cfg.D, dtype=tdt, device=device),
                "attn_out": torch.zeros(T, cfg.Hq, cfg.D, dtype=tdt, device=device),
            }
            self.aux = ev.LayerAux(*[self.a[n].data_ptr() for n, _ in ev.LayerAux._fields_])

    def run(self, layer: DeviceLayer):
        ev.evict_verify_layer(layer.ctx, layer.weights, self.tree_off, self.parent, self.B, self.T, self.k_cache,
                              self.v_cache, self.seq_stride, self.head_stride, self.ctx_len, self.max_ctx, self.x,
                              self.out, self.k_new, self.v_new, self.aux)

    def results(self) -> dict:
        torch.cuda.synchronize()
        r = {"out": to_host(self.out), "k_new": to_host(self.k_new), "v_new": to_host(self.v_new)}
        if self.aux is not None:
            r.update({k: to_host(v) for k, v in self.a.items()})
            r["union_count"] = int(r["union_count"][0])
        return r


def pack_lm_head(cfg, w_lm: np.ndarray, device="cuda:0") -> torch.Tensor:
    """Upload and pack W_lm [vocab, d] into the streaming layout."""
    raw = to_dev(w_lm, cfg.dtype, device)
    out = torch.empty_like(raw).reshape(-1)
    ev.evict_pack_dense(storage_code(cfg.dtype), raw, w_lm.shape[0], w_lm.shape[1], out)
    torch.cuda.synchronize()
    return out
