"""Multi-iteration speculative-decoding loop around the C entry points (host-side driver only).

One iteration = what the target side does between two calls of the draft model (Sec. 2.1 and
Sec. 3): EVICT prefix selection on the draft tree (optional), compaction of the kept nodes,
verification through the layer stack, LM head, acceptance, and the commit of the accepted
path to every layer's KV cache. Every step runs in the library's kernels; this module only
sequences the calls. Two ways of dispatching the selected length (Sec. 3.3):
  * host dispatch: two integers are read back per iteration (the selected length, by which the
    host sizes the verification launch -- the analogue of picking the pre-built graph for that
    length -- and the accepted length, which the drafter needs to go on);
  * device dispatch (`device_dispatch=True`): nothing is read back. The launches are sized for the
    whole draft tree and the kernels take the selected length from the selection's own output on
    the device (evict_dynamic_tokens); selected and accepted lengths of every iteration are kept
    in device logs. The host only tracks an upper bound of the context length (it grows by the tree
    size per iteration) until `resync()` reads the true one back; the whole iteration is one
    sequence of launches and can be captured as one graph.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import torch

from . import binding as ev


@dataclass
class DraftOnDevice:
    """One draft tree on the GPU (single sequence): CSR offsets, parents, draft probabilities,
    hidden states, draft token ids; target_next replaces the LM head's argmax when given (the
    synthetic drafter decides acceptance, see synth/drafter.py)."""
    tree_off: torch.Tensor
    parent: torch.Tensor
    q: torch.Tensor
    x: torch.Tensor
    tok: torch.Tensor
    target_next: Optional[torch.Tensor]
    n: int


@dataclass
class IterationLog:
    k_used: int
    path_len: int
    keep: Optional[List[int]] = None
    path: List[int] = field(default_factory=list)
    bonus: int = -1


class SpecLoop:
    def __init__(self, cfg, ctx, layers, k_caches, v_caches, seq_stride, head_stride, capacity, n_max,
                 lm_head=None, device="cuda:0", block_table=None, page_size=0, n_pages=0):
        """layers: list of LayerWeights; k_caches / v_caches: one [1][Hkv][capacity][D] tensor per layer;
        lm_head: (g_final, wlm_packed) or (g_final, wlm_packed, vocab) or None (then every draft must carry
        target_next); the vocabulary size is needed for acceptance under sampling.
        Paged caches: block_table int32 [1][pages] (pages for all `capacity` positions), page_size,
        n_pages; k_caches / v_caches are then the page pools [n_pages][Hkv][page_size][D] and
        seq_stride is the distance between pages."""
        self.cfg, self.ctx, self.layers = cfg, ctx, layers
        self.block_table, self.page_size, self.n_pages = block_table, page_size, n_pages
        self.kc, self.vc = k_caches, v_caches
        self.seq_stride, self.head_stride, self.capacity = seq_stride, head_stride, capacity
        self.n_max, self.lm_head = n_max, lm_head
        self.dtype_code = ev.EVICT_BF16 if cfg.dtype == "bf16" else ev.EVICT_F32
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.eb = 2 if cfg.dtype == "bf16" else 4
        i32, f32 = torch.int32, torch.float32
        N, L = n_max, len(layers)
        z = lambda *s, dt=i32: torch.zeros(*s, dtype=dt, device=device)  # noqa: E731
        self.k_star, self.keep, self.new_parent, self.new_off, self.est = z(1), z(N), z(N), z(2), z(1, dt=f32)
        self.xg, self.out = z(N, cfg.d, dt=tdt), z(N, cfg.d, dt=tdt)
        self.tokg, self.tng, self.next = z(N), z(N), z(N)
        self.k_new = [z(N, cfg.Hkv, cfg.D, dt=tdt) for _ in range(L)]
        self.v_new = [z(N, cfg.Hkv, cfg.D, dt=tdt) for _ in range(L)]
        self.path, self.path_len, self.bonus = z(1, N), z(1), z(1)
        # acceptance under sampling: full score rows of the LM head and the compacted per-node random numbers
        self.vocab = int(lm_head[2]) if (lm_head is not None and len(lm_head) > 2) else 0
        self.logits = z(N, self.vocab, dt=f32) if self.vocab else None
        self.ug = z(N, dt=f32)
        self.ctx_len = [z(1), z(1)]  # ping-pong: a commit reads one and writes the other
        self.cur = 0
        self.ctx_len_host = 0
        # device dispatch: per-iteration logs of the selected and the accepted length (ring of `log_slots` entries)
        self.log_slots = 1024
        self.k_log, self.plen_log = z(self.log_slots), z(self.log_slots)
        self.n_logged = 0

    def set_context_length(self, L: int):
        self.ctx_len[self.cur].fill_(L)
        self.ctx_len_host = L

    def resync(self) -> int:
        """Device dispatch: read the true context length back (one synchronising read) and drop the host's upper bound."""
        self.ctx_len_host = int(self.ctx_len[self.cur].item())
        return self.ctx_len_host

    def iteration_on_device(self, d: DraftOnDevice, cost: Optional[torch.Tensor], rho: Optional[float] = None) -> int:
        """One iteration with the selected length dispatched on the device: select -> gather -> stack -> LM head ->
        accept -> commit with no host read-back (greedy acceptance). Returns the log slot of this iteration
        (k_log / plen_log hold the selected and accepted lengths). Needs a cost table or rho (without a selection
        the length is the tree size and there is nothing to dispatch)."""
        if cost is None and rho is None:
            raise ValueError("device dispatch needs a selection (cost table or rho)")
        cfg, n = self.cfg, d.n
        slot = self.n_logged % self.log_slots
        k_star, plen = self.k_log[slot:slot + 1], self.plen_log[slot:slot + 1]
        cl_in, cl_out = self.ctx_len[self.cur], self.ctx_len[self.cur ^ 1]
        if cost is not None:
            ev.evict_select_prefix(None, d.tree_off, d.parent, d.q, 1, n, cost, n, k_star, self.keep, self.new_parent, self.new_off, self.est)
        else:
            ev.evict_select_prefix_coverage(None, d.tree_off, d.parent, d.q, 1, n, rho, n, k_star, self.keep, self.new_parent,
                                            self.new_off, self.est)
        ev.evict_gather_rows(d.x, self.xg, cfg.d * self.eb, d.tree_off, self.new_off, self.keep, 1, n)
        ev.evict_gather_rows(d.tok, self.tokg, 4, d.tree_off, self.new_off, self.keep, 1, n)
        if d.target_next is not None:
            ev.evict_gather_rows(d.target_next, self.tng, 4, d.tree_off, self.new_off, self.keep, 1, n)
        bound = max(self.ctx_len_host, 1)
        ev.evict_dynamic_tokens(self.ctx, self.new_off[1:])   # the count the kernels read: new_tree_off[B]
        try:
            if self.block_table is not None:
                ev.evict_verify_stack_paged(self.ctx, self.layers, self.new_off, self.new_parent, 1, n, self.kc, self.vc, self.seq_stride,
                                            self.head_stride, self.block_table, self.block_table.shape[-1], self.page_size, self.n_pages,
                                            cl_in, bound, self.xg, self.out, self.k_new, self.v_new)
            else:
                ev.evict_verify_stack(self.ctx, self.layers, self.new_off, self.new_parent, 1, n, self.kc, self.vc, self.seq_stride,
                                      self.head_stride, cl_in, bound, self.xg, self.out, self.k_new, self.v_new)
            tn = self.tng
            if self.lm_head is not None:
                ev.evict_lm_head_argmax(self.ctx, self.out, self.lm_head[0], self.lm_head[1], n, self.next)
                if d.target_next is None:
                    tn = self.next
        finally:
            ev.evict_dynamic_tokens(self.ctx, None)
        ev.evict_accept_path(None, self.new_off, self.new_parent, self.tokg, tn, 1, self.path, self.n_max, plen, self.bonus)
        if self.block_table is not None:
            ev.evict_kv_commit_stack_paged(self.ctx, self.dtype_code, cfg.Hkv, cfg.D, self.k_new, self.v_new, self.new_off, self.path,
                                           self.n_max, plen, self.kc, self.vc, self.seq_stride, self.head_stride, self.block_table,
                                           self.block_table.shape[-1], self.page_size, self.n_pages, cl_in, self.capacity, cl_out, 1)
        else:
            ev.evict_kv_commit_stack(self.ctx, self.dtype_code, cfg.Hkv, cfg.D, self.k_new, self.v_new, self.new_off, self.path,
                                     self.n_max, plen, self.kc, self.vc, self.seq_stride, self.head_stride, cl_in, self.capacity, cl_out, 1)
        self.cur ^= 1
        self.ctx_len_host = min(self.ctx_len_host + n, self.capacity)   # upper bound: at most n nodes are accepted
        self.n_logged += 1
        return slot

    def capture_on_device(self, d: DraftOnDevice, cost: Optional[torch.Tensor], rho: Optional[float] = None):
        """Record one device-dispatched iteration as a single HIP graph (call on a non-default torch stream).
        The tensors of `d` and `cost` are the graph's input buffers: refresh them in place before each
        evict_graph_launch. The context-length bound baked into the launches is the cache capacity, so every
        replay is covered; the new length is copied back into the buffer the graph reads, and every replay writes
        log slot 0 (k_log[0], plen_log[0])."""
        cur, logged = self.cur, self.n_logged
        self.n_logged = 0
        self.ctx_len_host = self.capacity
        ev.evict_graph_begin(self.ctx)
        try:
            self.iteration_on_device(d, cost, rho)
            self.ctx_len[cur].copy_(self.ctx_len[cur ^ 1])
        finally:
            graph = ev.evict_graph_end(self.ctx)
        self.cur, self.n_logged = cur, logged
        self.ctx_len_host = self.capacity
        return graph

    def iteration(self, d: DraftOnDevice, cost: Optional[torch.Tensor], log_lists: bool = False,
                  rho: Optional[float] = None, sample=None) -> IterationLog:
        """cost: device cost table float32[n + 1] -> EVICT truncation; rho -> the cost-agnostic
        coverage rule instead; neither -> verify all n nodes. sample = (temperature, u_node, u_bonus):
        acceptance by the sequential sibling rule under sampling (Sec. 2.1, Eq. 3) on the LM head's
        scores, with one random number per draft node (device float32[n], indexed like the nodes) and
        one per sequence; else the greedy rule."""
        if sample is not None and (self.lm_head is None or not self.vocab):
            raise ValueError("acceptance under sampling needs the LM head and its vocabulary size")
        cfg, n = self.cfg, d.n
        cl_in, cl_out = self.ctx_len[self.cur], self.ctx_len[self.cur ^ 1]
        if cost is not None or rho is not None:
            if cost is not None:
                ev.evict_select_prefix(None, d.tree_off, d.parent, d.q, 1, n, cost, n, self.k_star, self.keep,
                                       self.new_parent, self.new_off, self.est)
            else:
                ev.evict_select_prefix_coverage(None, d.tree_off, d.parent, d.q, 1, n, rho, n, self.k_star, self.keep,
                                                self.new_parent, self.new_off, self.est)
            k = int(self.k_star.item())
            ev.evict_gather_rows(d.x, self.xg, cfg.d * self.eb, d.tree_off, self.new_off, self.keep, 1, n)
            ev.evict_gather_rows(d.tok, self.tokg, 4, d.tree_off, self.new_off, self.keep, 1, n)
            if d.target_next is not None:
                ev.evict_gather_rows(d.target_next, self.tng, 4, d.tree_off, self.new_off, self.keep, 1, n)
            u_node = None
            if sample is not None:
                ev.evict_gather_rows(sample[1], self.ug, 4, d.tree_off, self.new_off, self.keep, 1, n)
                u_node = self.ug
            off, par, x, tok, tn = self.new_off, self.new_parent, self.xg, self.tokg, self.tng
        else:
            k = n
            off, par, x, tok, tn = d.tree_off, d.parent, d.x, d.tok, d.target_next
            u_node = sample[1] if sample is not None else None
        if self.block_table is not None:
            ev.evict_verify_stack_paged(self.ctx, self.layers, off, par, 1, k, self.kc, self.vc, self.seq_stride, self.head_stride,
                                        self.block_table, self.block_table.shape[-1], self.page_size, self.n_pages, cl_in,
                                        max(self.ctx_len_host, 1), x, self.out, self.k_new, self.v_new)
        else:
            ev.evict_verify_stack(self.ctx, self.layers, off, par, 1, k, self.kc, self.vc, self.seq_stride, self.head_stride,
                                  cl_in, max(self.ctx_len_host, 1), x, self.out, self.k_new, self.v_new)
        if sample is not None:
            ev.evict_lm_head_logits(self.ctx, self.out, self.lm_head[0], self.lm_head[1], k, self.logits)
            ev.evict_accept_path_sampled(self.ctx, off, par, tok, self.logits, self.vocab, sample[0], u_node, sample[2], 1, k,
                                         self.path, self.n_max, self.path_len, self.bonus)
        else:
            if self.lm_head is not None:
                ev.evict_lm_head_argmax(self.ctx, self.out, self.lm_head[0], self.lm_head[1], k, self.next)
            if d.target_next is None:
                tn = self.next
            ev.evict_accept_path(None, off, par, tok, tn, 1, self.path, self.n_max, self.path_len, self.bonus)
        if self.block_table is not None:
            ev.evict_kv_commit_stack_paged(self.ctx, self.dtype_code, cfg.Hkv, cfg.D, self.k_new, self.v_new, off, self.path,
                                           self.n_max, self.path_len, self.kc, self.vc, self.seq_stride, self.head_stride,
                                           self.block_table, self.block_table.shape[-1], self.page_size, self.n_pages, cl_in,
                                           self.capacity, cl_out, 1)
        else:
            ev.evict_kv_commit_stack(self.ctx, self.dtype_code, cfg.Hkv, cfg.D, self.k_new, self.v_new, off, self.path, self.n_max,
                                     self.path_len, self.kc, self.vc, self.seq_stride, self.head_stride, cl_in, self.capacity,
                                     cl_out, 1)
        plen = int(self.path_len.item())
        self.cur ^= 1
        self.ctx_len_host = min(self.ctx_len_host + plen, self.capacity)
        log = IterationLog(k_used=k, path_len=plen)
        if log_lists:
            log.keep = self.keep[:k].tolist() if (cost is not None or rho is not None) else None
            log.path = self.path[0, :plen].tolist()
            log.bonus = int(self.bonus.item())
        return log
