#!/usr/bin/env python3
"""Verify-step benchmark on one MI355X.

A step is one pass of the whole hot path over one batch of seeded synthetic input at the
Qwen3-30B-A3B-shaped configuration (one MoE decoder layer, bf16, KV context 2048, N = 32
draft-tree nodes): EVICT prefix selection on the draft probabilities, target-side tree
verification of the layer (tree-masked GQA attention, router top-k, expert union, grouped
SwiGLU expert GEMMs, combine) and greedy acceptance. Inputs are resident in HBM before the
timed region. Successive steps rotate over several copies of the layer's weights so the
last-level cache cannot hold the working set.

Prints one JSON line (metric = verify-step latency in microseconds) with the HBM roofline of
the dominant kernel (the gate/up grouped GEMM) measured by HIP events inside the library, and
the CPU oracle timed on the same inputs on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# the dominant kernel of the default workload (at most 32 tokens): contraction split over 8 wavefronts, bf16, one token
# tile, gate/up epilogue, two compile-time steps, non-temporal weight loads
GATEUP_KERNEL = "gemm_stream_kernel<BF16, 1, 8, 1, 2, true, 1, 2, true>"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--nodes", type=int, default=32, help="draft-tree size N")
    ap.add_argument("--ctx", type=int, default=2048, help="KV context length")
    ap.add_argument("--batch", type=int, default=1, help="sequences per call, each with its own tree of --nodes nodes")
    ap.add_argument("--ctx-max", type=int, default=0,
                    help="with --batch: context lengths drawn uniformly from [--ctx, --ctx-max] per sequence")
    ap.add_argument("--sigma", type=float, default=0.5, help="child = parent + sigma*N(0,1)")
    ap.add_argument("--copies", type=int, default=8,
                    help="weight copies rotated between steps (8: the projection weights of all copies, 308 MB, do not fit the "
                         "256 MB memory-side cache; with 4 they do and the projections read from it)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--seed", type=int, default=1000)
    ap.add_argument("--model", default="qwen3", choices=["qwen3", "dsv2lite", "qwen3_235b_tp8", "ling_flash2_tp4"],
                    help="layer shape; the default line is the Qwen3-30B-A3B-shaped one")
    ap.add_argument("--tune", action="append", default=[], help="key=value launch-shape knob (evict_tune)")
    ap.add_argument("--device-count", type=int, default=0, metavar="T",
                    help="on-device dispatch: the layer reads its token count (T, at most the tree size) from device memory "
                         "and the call passes the tree size as the upper bound (evict_dynamic_tokens)")
    ap.add_argument("--no-sweep", action="store_true",
                    help="default workload: leave the tree-size curve out (profiling runs: every launch is then the named workload)")
    ap.add_argument("--sweep", action="store_true",
                    help="not the default line: one JSON line per (N, sigma) point, N in 1..128, sigma in {0.2, 0.5, 1.0}")
    ap.add_argument("--cost", default="profile", choices=["profile", "surface"],
                    help="--loop: C(k) as profiled on the loop's own inputs, or collapsed from a cost surface over "
                         "(k, expert union) fitted to profiles at child noise 0.2 / the run's sigma / 1.0")
    ap.add_argument("--kv-page", type=int, default=0,
                    help="page size of a paged KV cache (power of two; pages assigned at random); 0 = contiguous caches")
    ap.add_argument("--launch", default="eager", choices=["graph", "eager"],
                    help="timed steps call the entry points (default), or replay one captured HIP graph per weight copy")
    ap.add_argument("--loop", action="store_true",
                    help="not the default line: multi-iteration speculative loop with a synthetic calibrated drafter, "
                         "fixed-size verification against EVICT truncation (one JSON line each)")
    ap.add_argument("--layers", type=int, default=0,
                    help="--loop / --stack: layers in the stack, distinct weights each (0: 8 for --loop; the model's depth for "
                         "--stack: 48 Qwen3-shaped, 27 DeepSeek-V2-Lite-shaped)")
    ap.add_argument("--stack", action="store_true",
                    help="not the default line: the whole target-side verification on the full-depth stack + LM head + acceptance, one "
                         "JSON line per point. Default: tree sizes 8..128 at child noise 0.2 and 1.0, ctx 4096; with --model "
                         "dsv2lite: N = 64, ctx 8192; with --batch B: B trees of --nodes nodes, contexts from [--ctx, --ctx-max], "
                         "cost table profiled on the device, the batch verified whole and truncated by the selection")
    ap.add_argument("--iters", type=int, default=128, help="--loop: timed iterations per mode")
    ap.add_argument("--probe-copy", type=int, default=0, metavar="MiB",
                    help="not the default line: run the plain copy and read kernels on MiB bytes (counter "
                         "calibration under rocprofv3 --pmc, and the streaming-read ceiling) and exit")
    return ap.parse_args()


def probe_copy(mib):
    """Plain copy / read kernels of a known size: what the HBM byte counters are scaled by."""
    import torch

    import paper_2605_00342_amd as ev

    n = mib * 1024 * 1024
    a = torch.empty(n, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    b = torch.empty_like(a)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    out = {"probe_bytes": n}
    for name, fn in (("copy", lambda: ev.evict_probe_copy(a, b, n)), ("read", lambda: ev.evict_probe_read(a, n, sink))):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        out[name + "_GBps"] = round((2 if name == "copy" else 1) * n / ms / 1e6, 1)
    print(json.dumps(out))


def sweep(args):
    """Latency, tokens/s and roofline fraction against tree size and union size (one layer)."""
    import torch

    import synth
    import paper_2605_00342_amd as ev
    from paper_2605_00342_amd import harness

    cfg = synth.CONFIGS["qwen3"]
    L = args.ctx
    base = synth.make_case("qwen3", n=128, L=L, seed=args.seed)
    layer = harness.DeviceLayer(cfg, base["W"], max_tokens=128, max_batch=1, max_ctx=L)
    names = ("wqkv", "wo", "wg", "w_gateup", "w_down")
    sets = [layer.weights]
    keep = []
    for _ in range(max(1, args.copies) - 1):
        cp = {n: getattr(layer, n).clone() for n in names}
        keep.append(cp)
        sets.append(ev.LayerWeights(layer.g_attn.data_ptr(), layer.g_moe.data_ptr(), cp["wqkv"].data_ptr(), cp["wo"].data_ptr(),
                                    cp["wg"].data_ptr(), cp["w_gateup"].data_ptr(), cp["w_down"].data_ptr(), None, None))
    eb = 2
    for sigma in (0.2, 0.5, 1.0):
        for N in (1, 8, 16, 32, 64, 128):
            g = synth.philox(args.seed, 100)
            par, q = synth.tree_eagle_style(N, g)
            case = dict(base)
            case.update(tree_off=np.array([0, N], np.int32), parent=par, parents=[par], q=q,
                        x=synth.hidden_states(par, cfg.d, sigma, synth.philox(args.seed, 300), cfg.dtype))
            dc = harness.DeviceCase(case, with_aux=True)
            dc.run(layer)
            U = int(dc.results()["union_count"])

            def step(i):
                ev.evict_verify_layer(layer.ctx, sets[i % len(sets)], dc.tree_off, dc.parent, 1, N, dc.k_cache, dc.v_cache,
                                      dc.seq_stride, dc.head_stride, dc.ctx_len, L, dc.x, dc.out, dc.k_new, dc.v_new, None)
            for i in range(args.warmup):
                step(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                step(i)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) * 1e6 / args.steps
            ns_bytes = U * 3 * cfg.d * cfg.F * eb + 2 * L * cfg.Hkv * cfg.D * eb
            print(json.dumps({"metric": "verify_layer_latency_us", "value": round(us, 2), "unit": "us", "nodes": N,
                              "sigma": sigma, "ctx": L, "union_experts": U, "tokens_per_s": round(N / us * 1e6, 1),
                              "north_star_bytes": ns_bytes,
                              "hbm_frac_north_star": round(ns_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}), flush=True)
    layer.close()


def spec_loop(args):
    """End-to-end simulated decoding: tokens/s and mean accepted tokens per iteration, verifying all
    N draft nodes every iteration against EVICT's cost-aware prefix (Sec. 3), on one stack of
    Qwen3-shaped layers + LM head. The cost table is profiled on the device (Sec. 3.2.3)."""
    import torch

    import synth
    import paper_2605_00342_amd as ev
    from paper_2605_00342_amd import harness
    from paper_2605_00342_amd.spec_loop import DraftOnDevice, SpecLoop

    dev = "cuda:0"
    cfg = synth.CONFIGS["qwen3"]
    N, L0, nl, vocab = args.nodes, args.ctx, args.layers or 8, 151936
    cap = L0 + 4096
    base = synth.make_case("qwen3", n=N, L=16, seed=args.seed)
    first = harness.DeviceLayer(cfg, base["W"], max_tokens=N, max_batch=1, max_ctx=cap, vocab=vocab)
    for kv in args.tune:
        key, val = kv.split("=")
        ev.evict_tune(first.ctx, key, int(val))
    # further layers: independent values of the same distribution, drawn directly in the packed layout
    # (packing is a permutation, so i.i.d. values packed or not are the same thing)
    gen = torch.Generator(device=dev).manual_seed(args.seed)
    keep, layers = [], [first.weights]
    for _ in range(nl - 1):
        cp = {n: (torch.randn(getattr(first, n).shape, generator=gen, device=dev) * 0.02).to(torch.bfloat16)
              for n in ("wqkv", "wo", "wg", "w_gateup", "w_down")}
        keep.append(cp)
        layers.append(ev.LayerWeights(first.g_attn.data_ptr(), first.g_moe.data_ptr(), cp["wqkv"].data_ptr(), cp["wo"].data_ptr(),
                                      cp["wg"].data_ptr(), cp["w_gateup"].data_ptr(), cp["w_down"].data_ptr(), None, None))
    wlm = (torch.randn(vocab * cfg.d, generator=gen, device=dev) * 0.02).to(torch.bfloat16)
    g_final = torch.ones(cfg.d, dtype=torch.bfloat16, device=dev)
    kc = [torch.randn(1, cfg.Hkv, cap, cfg.D, generator=gen, device=dev).to(torch.bfloat16) for _ in range(nl)]
    vc = [torch.randn(1, cfg.Hkv, cap, cfg.D, generator=gen, device=dev).to(torch.bfloat16) for _ in range(nl)]
    loop = SpecLoop(cfg, first.ctx, layers, kc, vc, cfg.Hkv * cap * cfg.D, cap * cfg.D, cap, N, lm_head=(g_final, wlm))

    pool = []
    for it in range(64):
        d = synth.draft_iteration(cfg, N, args.seed, it, args.sigma, vocab)
        pool.append(DraftOnDevice(harness.dev_i32(np.array([0, N])), harness.dev_i32(d["parent"]), torch.from_numpy(d["q"]).to(dev),
                                  harness.to_dev(d["x"], cfg.dtype), harness.dev_i32(d["tok"]), harness.dev_i32(d["target_next"]), N))

    # cost table C(k) of the stack, timed on the device stream; the LM head's share is constant in k
    # up to its token tiles and is left out, as the layers are what grows with k
    d0 = pool[0]
    loop.set_context_length(L0)
    surface = None
    if args.cost == "profile":
        cost = ev.evict_profile_cost(first.ctx, layers, d0.tree_off, d0.parent, N, kc, vc, cap * cfg.D, loop.ctx_len[loop.cur], L0,
                                     d0.x, loop.out, loop.k_new, loop.v_new, 6)
    else:
        # points (k, mean union, ms) at three routing spreads; C(k) = surface at the union this run's inputs show
        from paper_2605_00342_amd import cost_model as cm
        sets = []
        for sg in (0.2, args.sigma, 1.0):
            dd = synth.draft_iteration(cfg, N, args.seed, 0, sg, vocab)
            sets.append(dict(tree_off=d0.tree_off, parent=harness.dev_i32(dd["parent"]), k_caches=kc, v_caches=vc,
                             kv_head_stride=cap * cfg.D, ctx_len=loop.ctx_len[loop.cur], max_ctx_host=L0,
                             x_in=harness.to_dev(dd["x"], cfg.dtype), x_out=loop.out, k_new=loop.k_new, v_new=loop.v_new))
        ks_, us_, ts_, _ = cm.profile_cost_surface(first.ctx, layers, sets, N, 6)
        coef, rms = cm.fit_cost_surface(ks_, us_, ts_)
        own_union = [0.0] + [float(u) for u in us_[N:2 * N]]
        cost = [float(c) for c in cm.collapse_cost(coef, N, cfg.E, cfg.k, own_union)]
        surface = {"ms = a + b*k + c*union": [round(float(c), 6) for c in coef], "rms_residual_ms": round(rms, 5),
                   "points": int(ks_.size), "union_at_k": [round(u, 2) for u in own_union[1:]],
                   "union_range_at_N": [round(float(us_[N - 1]), 2), round(float(us_[3 * N - 1]), 2)]}
    results = {}
    cost_dev = None
    # plain autoregressive decoding for comparison: a one-node tree per iteration (the root alone: one token each)
    pool1 = [DraftOnDevice(harness.dev_i32(np.array([0, 1])), p.parent[:1], p.q[:1], p.x[:1], p.tok[:1], p.target_next[:1], 1)
             for p in pool]
    for mode in ("autoregressive", "verify_all", "evict", "evict_device_dispatch", "coverage_0.7", "coverage_0.4"):
        rho = float(mode.split("_")[1]) if mode.startswith("coverage") else None
        drafts = pool1 if mode == "autoregressive" else pool
        if mode == "evict":
            # C(k) must be the cost of a whole iteration at length k: the part outside the layer stack
            # (LM head, acceptance, commits, read-backs) is taken from the measured full-size iteration
            offset = max(results["verify_all"]["ms_per_iteration"] - cost[N], 0.0)
            cost = [c + offset for c in cost]
            cost_dev = torch.tensor(cost, dtype=torch.float32, device=dev)
        table = cost_dev if mode in ("evict", "evict_device_dispatch") else None
        if mode == "evict_device_dispatch":
            # Sec. 3.3: the selected length is dispatched on the device. Launches are sized for the whole tree, the
            # kernels read the selected length from the selection's output, nothing is read back inside an
            # iteration; the host refreshes its upper bound of the context length every 16 iterations.
            assert args.iters <= loop.log_slots, "--iters exceeds the loop's device log"
            loop.set_context_length(L0)
            for i in range(8):
                loop.iteration_on_device(drafts[i % len(drafts)], table)
            loop.set_context_length(L0)
            loop.n_logged = 0
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.iters):
                loop.iteration_on_device(drafts[i % len(drafts)], table)
                if (i + 1) % 16 == 0:
                    loop.resync()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            tokens = int(loop.plen_log[:args.iters].sum().item())
            ksum = int(loop.k_log[:args.iters].sum().item())
            results[mode] = {"tokens_per_s": tokens / dt, "ms_per_iteration": dt * 1e3 / args.iters,
                             "mean_accepted_tokens": tokens / args.iters, "mean_verified_nodes": ksum / args.iters}
            continue
        loop.set_context_length(L0)
        for i in range(8):
            loop.iteration(drafts[i % len(drafts)], table, rho=rho)
        loop.set_context_length(L0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tokens = ksum = 0
        for i in range(args.iters):
            log = loop.iteration(drafts[i % len(drafts)], table, rho=rho)
            tokens += log.path_len
            ksum += log.k_used
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        results[mode] = {"tokens_per_s": tokens / dt, "ms_per_iteration": dt * 1e3 / args.iters,
                         "mean_accepted_tokens": tokens / args.iters, "mean_verified_nodes": ksum / args.iters}
    for mode, r in results.items():
        print(json.dumps({"metric": "simulated_decode_tokens_per_s", "mode": mode, "value": round(r["tokens_per_s"], 1),
                          "unit": "tokens/s", "ms_per_iteration": round(r["ms_per_iteration"], 4),
                          "mean_accepted_tokens": round(r["mean_accepted_tokens"], 3),
                          "mean_verified_nodes": round(r["mean_verified_nodes"], 2),
                          "speedup_vs_verify_all": round(r["tokens_per_s"] / results["verify_all"]["tokens_per_s"], 4),
                          "speedup_vs_autoregressive": round(r["tokens_per_s"] / results["autoregressive"]["tokens_per_s"], 4),
                          "config": {"workload": f"qwen3-30b-a3b-shaped stack of {nl} layers + LM head, N={N} draft nodes, "
                                                 f"ctx from {L0}, synthetic calibrated drafter, sigma={args.sigma}",
                                     "iterations": args.iters},
                          "cost_table_ms": [round(c, 4) for c in cost[1:]] if mode == "evict" else None,
                          "cost_surface": surface if mode == "evict" else None,
                          "data": "synthetic", "dtype": "bf16"}), flush=True)
    first.close()


def stack_bench(args, collect=None):
    """(collect: a list that takes the records instead of stdout.) The whole target-side verification at full depth: layer stack, LM head + argmax, greedy acceptance
    (and, for a batch, EVICT's selection and the row gather in front of it), against tree size and child
    noise. Weights of the layers after the first are independent draws made directly in the packed layout
    (packing is a permutation, so the distribution is the same); caches are N(0, 1)."""
    import torch

    import synth
    import paper_2605_00342_amd as ev
    from paper_2605_00342_amd import harness

    dev = "cuda:0"
    cfg = synth.CONFIGS[args.model]
    nl = args.layers or {"qwen3": 48, "dsv2lite": 27}.get(args.model, 8)
    vocab, B = 151936, args.batch
    batched = B > 1
    if batched:
        L_list = [int(v) for v in synth.philox(args.seed, 950).integers(args.ctx, max(args.ctx_max, args.ctx) + 1, B)]
        points = [(args.nodes, args.sigma)]
    elif args.model == "dsv2lite":
        L_list, points = [8192 if args.ctx == 2048 else args.ctx], [(64, args.sigma)]
    else:
        L_list = [4096 if args.ctx == 2048 else args.ctx]
        points = [(n, s) for s in (0.2, 1.0) for n in (8, 16, 32, 64, 128)]
    L = max(L_list)
    n_max = max(n for n, _ in points)
    T_max = n_max * B
    tree = "bfs" if (args.model == "dsv2lite" or batched) else "eagle"
    base = synth.make_case(args.model, n=n_max, L=16, seed=args.seed, tree=tree)
    first = harness.DeviceLayer(cfg, base["W"], max_tokens=T_max, max_batch=B, max_ctx=L, vocab=vocab)
    for kv in args.tune:
        key, val = kv.split("=")
        ev.evict_tune(first.ctx, key, int(val))
    gen = torch.Generator(device=dev).manual_seed(args.seed)
    names = ["wqkv", "wo", "wg", "w_gateup", "w_down"] + (["ws_gateup", "ws_down"] if cfg.n_shared else [])
    keep, layers = [], [first.weights]
    for _ in range(nl - 1):
        cp = {n: (torch.randn(getattr(first, n).shape, generator=gen, device=dev) * 0.02).to(torch.bfloat16) for n in names}
        keep.append(cp)
        layers.append(ev.LayerWeights(first.g_attn.data_ptr(), first.g_moe.data_ptr(), cp["wqkv"].data_ptr(), cp["wo"].data_ptr(),
                                      cp["wg"].data_ptr(), cp["w_gateup"].data_ptr(), cp["w_down"].data_ptr(),
                                      cp["ws_gateup"].data_ptr() if cfg.n_shared else None,
                                      cp["ws_down"].data_ptr() if cfg.n_shared else None))
    wlm = (torch.randn(vocab * cfg.d, generator=gen, device=dev) * 0.02).to(torch.bfloat16)
    g_final = torch.ones(cfg.d, dtype=torch.bfloat16, device=dev)
    kc = [torch.randn(B, cfg.Hkv, L, cfg.D, generator=gen, device=dev).to(torch.bfloat16) for _ in range(nl)]
    vc = [torch.randn(B, cfg.Hkv, L, cfg.D, generator=gen, device=dev).to(torch.bfloat16) for _ in range(nl)]
    seq_stride, head_stride = cfg.Hkv * L * cfg.D, L * cfg.D
    ctx_len = harness.dev_i32(np.array(L_list))
    i32, f32, bf = torch.int32, torch.float32, torch.bfloat16
    out = torch.zeros(T_max, cfg.d, dtype=bf, device=dev)
    k_new = [torch.zeros(T_max, cfg.Hkv, cfg.D, dtype=bf, device=dev) for _ in range(nl)]
    v_new = [torch.zeros(T_max, cfg.Hkv, cfg.D, dtype=bf, device=dev) for _ in range(nl)]
    nxt = torch.zeros(T_max, dtype=i32, device=dev)
    path = torch.zeros(B, 16, dtype=i32, device=dev)
    plen, bonus = torch.zeros(B, dtype=i32, device=dev), torch.zeros(B, dtype=i32, device=dev)
    eb = 2
    expert_bytes = 3 * cfg.d * cfg.F * eb
    kv_bytes = 2 * int(sum(L_list)) * cfg.Hkv * cfg.D * eb
    proj_bytes = (2 * cfg.Hq * cfg.D * cfg.d + 2 * cfg.Hkv * cfg.D * cfg.d) * eb + cfg.E * cfg.d * eb
    lm_bytes = vocab * cfg.d * eb

    def measure(fn, reps):
        """ms per call and mean union per layer over `reps` timed calls."""
        for _ in range(3):
            fn()
        ev.evict_union_total(first.ctx, reset=True)
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / reps
        return ms, ev.evict_union_total(first.ctx, reset=True) / (reps * nl)

    def record(what, ms, U, T, extra):
        ns = nl * ((U + cfg.n_shared) * expert_bytes + kv_bytes)
        rec = {"metric": "verify_stack_latency_ms", "value": round(ms, 4), "unit": "ms", "what": what,
               "tokens_per_s": round(T / ms * 1e3, 1), "us_per_layer": round(ms * 1e3 / nl, 2),
               "mean_union_per_layer": round(U, 2), "north_star_bytes": int(ns),
               "hbm_frac_north_star": round(ns / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
               "hbm_frac_all_required": round((ns + nl * proj_bytes + lm_bytes) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
               **extra, "config": {"workload": f"{WORKLOAD_NAMES[args.model]}-shaped stack of {nl} layers + LM head "
                                               f"({vocab} rows) + greedy acceptance, ctx={L_list}",
                                   "layers": nl}, "data": "synthetic", "dtype": "bf16"}
        if collect is not None:
            collect.append(rec)
        else:
            print(json.dumps(rec), flush=True)

    reps = max(args.steps // 10, 5)
    if not batched:
        for N, sigma in points:
            g = synth.philox(args.seed, 100)
            if tree == "eagle":
                par, q = synth.tree_eagle_style(N, g)
            else:
                par = synth.tree_bfs_random(N, g)
            x = harness.to_dev(synth.hidden_states(par, cfg.d, sigma, synth.philox(args.seed, 300), cfg.dtype), cfg.dtype)
            toff, pard = harness.dev_i32(np.array([0, N])), harness.dev_i32(par)
            tok = harness.dev_i32(synth.philox(args.seed, 900).integers(0, vocab, N).astype(np.int32))

            def verify():
                ev.evict_verify_stack(first.ctx, layers, toff, pard, 1, N, kc, vc, seq_stride, head_stride, ctx_len, L, x, out,
                                      k_new, v_new)
                ev.evict_lm_head_argmax(first.ctx, out, g_final, wlm, N, nxt, None, None)
                ev.evict_accept_path(None, toff, pard, tok, nxt, 1, path, 16, plen, bonus)
            ms, U = measure(verify, reps)
            record("verify all nodes", ms, U, N, {"nodes": N, "sigma": sigma})
        first.close()
        return

    # a batch: the whole step first, then the cost table profiled on the device, then the step truncated by the selection
    N = args.nodes
    case = synth.make_case(args.model, n=N, L=16, seed=args.seed, sigma=args.sigma, batch=B, L_list=[16] * B, tree="bfs")
    T = int(case["tree_off"][-1])
    x = harness.to_dev(case["x"], cfg.dtype)
    toff, pard = harness.dev_i32(case["tree_off"]), harness.dev_i32(case["parent"])
    q_dev = torch.from_numpy(case["q"]).to(dev)
    tok = harness.dev_i32(synth.philox(args.seed, 900).integers(0, vocab, T).astype(np.int32))
    def whole():
        ev.evict_verify_stack(first.ctx, layers, toff, pard, B, T, kc, vc, seq_stride, head_stride, ctx_len, L, x, out, k_new, v_new)
        ev.evict_lm_head_argmax(first.ctx, out, g_final, wlm, T, nxt, None, None)
        ev.evict_accept_path(None, toff, pard, tok, nxt, B, path, 16, plen, bonus)
    ms_all, U_all = measure(whole, reps)

    # Cost table on the device (Sec. 3.2.3; App. C.5 applies the same rule per sequence of a batch): C(k) = latency
    # of this batch's whole step (stack, LM head, acceptance) when every tree is cut to its first k nodes (parents
    # precede children, so those are a tree), timed with events on the stream; the mean union per layer beside it
    cost, umean = [0.0], [0.0]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    off_h = case["tree_off"]
    for k in range(1, N + 1):
        rows = np.concatenate([np.arange(off_h[b], off_h[b] + k) for b in range(B)])
        rd = torch.from_numpy(rows).to(dev)
        xk, pk_, tk = x[rd].contiguous(), pard[rd].contiguous(), tok[rd].contiguous()
        ok = harness.dev_i32(np.arange(B + 1) * k)

        def cut():
            ev.evict_verify_stack(first.ctx, layers, ok, pk_, B, B * k, kc, vc, seq_stride, head_stride, ctx_len, L, xk, out, k_new, v_new)
            ev.evict_lm_head_argmax(first.ctx, out, g_final, wlm, B * k, nxt, None, None)
            ev.evict_accept_path(None, ok, pk_, tk, nxt, B, path, 16, plen, bonus)
        cut()
        ev.evict_union_total(first.ctx, reset=True)
        e0.record()
        for _ in range(3):
            cut()
        e1.record()
        torch.cuda.synchronize()
        cost.append(e0.elapsed_time(e1) / 3)
        umean.append(ev.evict_union_total(first.ctx, reset=True) / (3 * nl))
    cost[0] = cost[1]
    cost_dev = torch.tensor(cost, dtype=f32, device=dev)
    ks = torch.zeros(B, dtype=i32, device=dev); keepn = torch.zeros(T, dtype=i32, device=dev)
    npar = torch.zeros(T, dtype=i32, device=dev); noff = torch.zeros(B + 1, dtype=i32, device=dev)
    est = torch.zeros(B, dtype=f32, device=dev); order = torch.zeros(T, dtype=i32, device=dev)
    psum = torch.zeros(T, dtype=f32, device=dev)
    x2, tok2 = torch.zeros_like(x), torch.zeros_like(tok)
    ev.evict_select_prefix(None, toff, pard, q_dev, B, T, cost_dev, N, ks, keepn, npar, noff, est, order, psum)
    torch.cuda.synchronize()
    T2 = int(noff[B].item())   # outside the timed region: sizes the launches of the truncated step

    def truncated():
        ev.evict_select_prefix(None, toff, pard, q_dev, B, T, cost_dev, N, ks, keepn, npar, noff, est, order, psum)
        ev.evict_gather_rows(x, x2, cfg.d * eb, toff, noff, keepn, B, T)
        ev.evict_gather_rows(tok, tok2, 4, toff, noff, keepn, B, T)
        ev.evict_verify_stack(first.ctx, layers, noff, npar, B, T2, kc, vc, seq_stride, head_stride, ctx_len, L, x2, out, k_new, v_new)
        ev.evict_lm_head_argmax(first.ctx, out, g_final, wlm, T2, nxt, None, None)
        ev.evict_accept_path(None, noff, npar, tok2, nxt, B, path, 16, plen, bonus)
    ms_tr, U_tr = measure(truncated, reps)
    # expected accepted tokens of a step (Eq. 8): the sum of the kept nodes' scores, per sequence, summed over the batch
    ps, ksh, off_h = psum.cpu().numpy(), ks.cpu().numpy(), case["tree_off"]
    s_full = float(sum(ps[off_h[b + 1] - 1] for b in range(B)))
    s_kept = float(sum(ps[off_h[b] + int(ksh[b]) - 1] for b in range(B)))
    common = {"sequences": B, "nodes_per_tree": N, "sigma": args.sigma,
              "cost_table_ms": [round(c, 4) for c in cost[1:]], "profiled_union_at_k": [round(u, 2) for u in umean[1:]]}
    record("batch verified whole", ms_all, U_all, T, {**common, "verified_nodes": T, "expected_accepted_tokens": round(s_full, 3),
                                                      "expected_accepted_tokens_per_s": round(s_full / ms_all * 1e3, 1)})
    record("batch truncated by the selection (Eq. 10), selection and gather inside the timed step", ms_tr, U_tr, T2,
           {**common, "verified_nodes": T2, "k_star": [int(v) for v in ksh], "expected_accepted_tokens": round(s_kept, 3),
            "expected_accepted_tokens_per_s": round(s_kept / ms_tr * 1e3, 1),
            "speedup_in_expected_tokens_per_s": round((s_kept / ms_tr) / (s_full / ms_all), 4)})
    first.close()


WORKLOAD_NAMES = {"qwen3": "qwen3-30b-a3b", "dsv2lite": "deepseek-v2-lite",
                  "qwen3_235b_tp8": "qwen3-235b-a22b (one rank of TP=8)",
                  "ling_flash2_tp4": "ling-flash-2.0 (one rank of TP=4)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    import synth
    import paper_2605_00342_amd as ev
    from paper_2605_00342_amd import harness

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.probe_copy:
        probe_copy(args.probe_copy)
        return
    if args.sweep:
        sweep(args)
        return
    if args.loop:
        spec_loop(args)
        return
    if args.stack:
        stack_bench(args)
        return
    cfg = synth.CONFIGS[args.model]
    N, L, B = args.nodes, args.ctx, args.batch
    L_list = None
    if B > 1:
        gl = synth.philox(args.seed, 950)
        L_list = [int(v) for v in gl.integers(L, max(args.ctx_max, L) + 1, B)]
        L = max(L_list)
    case = synth.make_case(args.model, n=N, L=L, seed=args.seed, sigma=args.sigma, batch=B, L_list=L_list,
                           tree="auto" if args.model == "dsv2lite" else "eagle")
    T = int(case["tree_off"][-1])
    default_workload = (B == 1 and args.model == "qwen3" and not args.kv_page and not args.tune and args.launch == "eager"
                        and not args.device_count and (N, L, args.sigma) == (32, 2048, 0.5))
    layer = harness.DeviceLayer(cfg, case["W"], max_tokens=max(T, 128) if default_workload else T, max_batch=B, max_ctx=L)
    dc = harness.DeviceCase(case, with_aux=True)
    for kv in args.tune:
        key, val = kv.split("=")
        ev.evict_tune(layer.ctx, key, int(val))
    if args.device_count:
        if B != 1:
            sys.exit("bench.py --device-count: one sequence only")
        # the first `count` nodes of a topologically numbered tree are a tree: offsets and the device word agree on it
        count_dev = torch.tensor([min(args.device_count, T)], dtype=torch.int32, device="cuda:0")
        dc.tree_off = torch.tensor([0, min(args.device_count, T)], dtype=torch.int32, device="cuda:0")
        ev.evict_dynamic_tokens(layer.ctx, count_dev)

    # weight copies (same values, distinct addresses) so that no step finds its weights in cache
    names = ("wqkv", "wo", "wg", "w_gateup", "w_down")
    weight_sets = [layer.weights]
    keep_alive = []
    for _ in range(max(1, args.copies) - 1):
        cp = {n: getattr(layer, n).clone() for n in names}
        if cfg.n_shared:
            cp["ws_gateup"], cp["ws_down"] = layer.ws_gateup.clone(), layer.ws_down.clone()
        keep_alive.append(cp)
        weight_sets.append(ev.LayerWeights(layer.g_attn.data_ptr(), layer.g_moe.data_ptr(), cp["wqkv"].data_ptr(),
                                           cp["wo"].data_ptr(), cp["wg"].data_ptr(), cp["w_gateup"].data_ptr(),
                                           cp["w_down"].data_ptr(),
                                           cp["ws_gateup"].data_ptr() if cfg.n_shared else None,
                                           cp["ws_down"].data_ptr() if cfg.n_shared else None))

    # selection / acceptance inputs
    i32, f32 = torch.int32, torch.float32
    q_dev = torch.from_numpy(case["q"]).to(dev)
    cost = synth.cost_linear_in_union(N, cfg.E, cfg.k)
    cost_dev = torch.from_numpy(cost).to(dev)
    sel = dict(k_star=torch.zeros(B, dtype=i32, device=dev), keep=torch.zeros(T, dtype=i32, device=dev),
               new_parent=torch.zeros(T, dtype=i32, device=dev), new_off=torch.zeros(B + 1, dtype=i32, device=dev),
               est=torch.zeros(B, dtype=f32, device=dev))
    g = synth.philox(args.seed, 900)
    target_next = g.integers(0, 151936, T).astype(np.int32)
    draft_tok = np.concatenate([synth.plant_draft_tokens(p, target_next[o:o + len(p)], 151936, g)
                                for p, o in zip(case["parents"], case["tree_off"][:-1])])
    tn_dev, dt_dev = harness.dev_i32(target_next), harness.dev_i32(draft_tok)
    path = torch.zeros(B, N, dtype=i32, device=dev)
    path_len = torch.zeros(B, dtype=i32, device=dev)
    bonus = torch.zeros(B, dtype=i32, device=dev)

    paged = None
    if args.kv_page:
        # the same cache contents scattered over randomly assigned pages; read through a block table
        P = args.kv_page
        pk, pv, table, n_pages = synth.to_pages(case["K"], case["V"], P, [int(v) for v in case["ctx_len"]],
                                                synth.philox(args.seed, 960))
        paged = dict(pk=harness.to_dev(pk, cfg.dtype), pv=harness.to_dev(pv, cfg.dtype), table=harness.dev_i32(table),
                     stride=table.shape[1], n_pages=n_pages, P=P)

    def layer_call(i):
        w = weight_sets[i % len(weight_sets)]
        if paged:
            ev.evict_verify_stack_paged(layer.ctx, [w], dc.tree_off, dc.parent, B, T, [paged["pk"]], [paged["pv"]],
                                        cfg.Hkv * paged["P"] * cfg.D, paged["P"] * cfg.D, paged["table"], paged["stride"],
                                        paged["P"], paged["n_pages"], dc.ctx_len, L, dc.x, dc.out, [dc.k_new], [dc.v_new])
        else:
            ev.evict_verify_layer(layer.ctx, w, dc.tree_off, dc.parent, B, T, dc.k_cache, dc.v_cache, dc.seq_stride,
                                  dc.head_stride, dc.ctx_len, L, dc.x, dc.out, dc.k_new, dc.v_new, None)

    def step(i):
        ev.evict_select_prefix(None, dc.tree_off, dc.parent, q_dev, B, T, cost_dev, N, sel["k_star"], sel["keep"],
                               sel["new_parent"], sel["new_off"], sel["est"])
        layer_call(i)
        ev.evict_accept_path(None, dc.tree_off, dc.parent, dt_dev, tn_dev, B, path, N, path_len, bonus)

    # one checked run: union size for the byte count
    dc.run(layer)
    res = dc.results()
    U = int(res["union_count"])

    def timed(fn):
        for i in range(args.warmup):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    def spread(fn, batches=20):
        """p10 / p50 / p90 of the mean step time over batches of steps (outside the timed region)."""
        per = max(args.steps // batches, 1)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(batches + 1)]
        evs[0].record()
        for b in range(batches):
            for i in range(per):
                fn(b * per + i)
            evs[b + 1].record()
        torch.cuda.synchronize()
        t = sorted(evs[b].elapsed_time(evs[b + 1]) * 1e3 / per for b in range(batches))
        return [round(t[int(q * (batches - 1))], 2) for q in (0.1, 0.5, 0.9)]

    other_ms = None
    if args.launch == "graph":
        # one graph per weight copy: the same three calls, recorded once on a side stream
        side = torch.cuda.Stream()
        graphs = []
        with torch.cuda.stream(side):
            for i in range(len(weight_sets)):
                ev.evict_graph_begin(layer.ctx)
                step(i)
                graphs.append(ev.evict_graph_end(layer.ctx))

            def replay(i):
                ev.evict_graph_launch(graphs[i % len(graphs)])

            ms_per_step = timed(replay)
        torch.cuda.synchronize()
        other_ms = timed(step)  # the same steps as direct calls, for comparison
        for gr in graphs:
            ev.evict_graph_destroy(gr)
    else:
        ms_per_step = timed(step)

    # per-stage durations from HIP events recorded by the library on the launch stream
    ev.evict_stage_timing(layer.ctx, True)
    stage_ms = {n: 0.0 for n in ev.STAGES}
    n_timed = min(args.steps, 50)
    for i in range(n_timed):
        step(i)
        t = ev.evict_stage_times(layer.ctx)
        for n in ev.STAGES:
            stage_ms[n] += t[n] / n_timed
    ev.evict_stage_timing(layer.ctx, False)

    # The same layer calls without the stage events, between two events on the launch stream: what
    # the stage events add per stage is (sum of stage times - this) / stages. (An event pair around
    # nothing, like the empty "shared" stage, costs more than an event between two kernels does.)
    layer_only = layer_call
    for i in range(5):
        layer_only(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(n_timed):
        layer_only(i)
    e1.record()
    torch.cuda.synchronize()
    layer_ms = e0.elapsed_time(e1) / n_timed

    eb = 2
    expert_bytes = 3 * cfg.d * cfg.F * eb
    kv_bytes = 2 * int(np.sum(case["ctx_len"])) * cfg.Hkv * cfg.D * eb
    proj_bytes = (2 * cfg.Hq * cfg.D * cfg.d + 2 * cfg.Hkv * cfg.D * cfg.d) * eb + cfg.E * cfg.d * eb
    north_star_bytes = (U + cfg.n_shared) * expert_bytes + kv_bytes
    all_bytes = north_star_bytes + proj_bytes
    # algorithmic bytes of the dominant kernel per launch (shared experts ride in the same launch)
    gateup_bytes = (U + cfg.n_shared) * 2 * cfg.d * cfg.F * eb
    ev_overhead_ms = max(sum(stage_ms.values()) - layer_ms, 0.0) / len(ev.STAGES)
    gateup_ms = max(stage_ms["gateup"] - ev_overhead_ms, 1e-6)
    gateup_s = gateup_ms * 1e-3
    achieved = gateup_bytes / gateup_s / 1e9
    # HBM bytes per launch of that kernel by hardware counters: not measurable from inside this process; taken from the
    # committed rocprofv3 --pmc summary of this same command when it was made for this workload and this kernel
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    if os.path.exists(tpath) and default_workload and args.sigma == 0.5:
        try:
            rec = json.load(open(tpath)).get(f"gateup_N{N}_L{L}")
            if isinstance(rec, dict) and rec.get("kernel") == GATEUP_KERNEL:
                traffic, traffic_source = rec["bytes_per_launch"], rec.get("source")
        except Exception:
            traffic = None

    out = {
        "metric": "verify_step_latency_us",
        "value": round(ms_per_step * 1e3, 2),
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{WORKLOAD_NAMES[args.model]}-shaped MoE layer, N={N} tree nodes, ctx={L if B == 1 else [int(v) for v in case['ctx_len']]}, {B} sequence{'s' if B > 1 else ''}, sigma={args.sigma}",
                   "d_model": cfg.d, "heads": f"{cfg.Hq}q/{cfg.Hkv}kv x {cfg.D}", "experts": f"{cfg.E} top-{cfg.k}",
                   "d_ff": cfg.F, "union_experts": U, "weight_copies": len(weight_sets)},
        "step_us_p10_p50_p90": spread(step),
        "launch": args.launch,
        "eager_us": None if other_ms is None else round(other_ms * 1e3, 2),
        "tokens_per_s": round(T / (ms_per_step * 1e-3), 1),
        "step_roofline": {"north_star_bytes": north_star_bytes, "all_required_bytes": all_bytes,
                          "hbm_frac_north_star": round(north_star_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                          "hbm_frac_all_required": round(all_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "stage_us": {n: round(v * 1e3, 2) for n, v in stage_ms.items()},
        "roofline": {"bound": "hbm", "kernel": GATEUP_KERNEL + " (gate/up grouped GEMM + SiLU gating)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
                     "bytes_per_launch": gateup_bytes, "avg_launch_us": round(gateup_ms * 1e3, 2),
                     "event_overhead_us": round(ev_overhead_ms * 1e3, 2), "layer_us": round(layer_ms * 1e3, 2)},
    }

    # streaming-read ceiling of this device, measured in the same run (plain read kernel, 1 GiB, non-temporal loads)
    nprobe = 1 << 30
    pa = torch.empty(nprobe, dtype=torch.uint8, device=dev).random_(0, 255)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    for _ in range(2):
        ev.evict_probe_read(pa, nprobe, sink)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        ev.evict_probe_read(pa, nprobe, sink)
    e1.record()
    torch.cuda.synchronize()
    ceiling = 5 * nprobe / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del pa
    out["read_ceiling_GBps"] = round(ceiling, 1)
    out["roofline"]["frac_of_read_ceiling"] = round(achieved / ceiling, 4)
    out["step_roofline"]["frac_of_read_ceiling_north_star"] = round(north_star_bytes / (ms_per_step * 1e-3) / 1e9 / ceiling, 4)

    # the metric's curve: the same step against the tree size N (same layer, context and child noise)
    if default_workload and not args.no_sweep:
        pts = []
        for Ns in (8, 16, 32, 64, 128):
            if Ns == N:
                pts.append({"nodes": N, "us": round(ms_per_step * 1e3, 2), "union_experts": U,
                            "hbm_frac_north_star": round(north_star_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                            "tokens_per_s": round(N / (ms_per_step * 1e-3), 1)})
                continue
            gs = synth.philox(args.seed, 100)
            par, q = synth.tree_eagle_style(Ns, gs)
            cs = dict(case)
            cs.update(tree_off=np.array([0, Ns], np.int32), parent=par, parents=[par], q=q,
                      x=synth.hidden_states(par, cfg.d, args.sigma, synth.philox(args.seed, 300), cfg.dtype))
            ds = harness.DeviceCase(cs, with_aux=True)
            ds.run(layer)
            Us = int(ds.results()["union_count"])
            qd = torch.from_numpy(q).to(dev)
            cd = torch.from_numpy(synth.cost_linear_in_union(Ns, cfg.E, cfg.k)).to(dev)
            tn = harness.dev_i32(g.integers(0, 151936, Ns).astype(np.int32))
            dt = harness.dev_i32(g.integers(0, 151936, Ns).astype(np.int32))
            pth = torch.zeros(1, Ns, dtype=i32, device=dev)
            sel_s = dict(k_star=torch.zeros(1, dtype=i32, device=dev), keep=torch.zeros(Ns, dtype=i32, device=dev),
                         new_parent=torch.zeros(Ns, dtype=i32, device=dev), new_off=torch.zeros(2, dtype=i32, device=dev),
                         est=torch.zeros(1, dtype=f32, device=dev))

            def step_s(i):
                ev.evict_select_prefix(None, ds.tree_off, ds.parent, qd, 1, Ns, cd, Ns, sel_s["k_star"], sel_s["keep"], sel_s["new_parent"],
                                       sel_s["new_off"], sel_s["est"])
                ev.evict_verify_layer(layer.ctx, weight_sets[i % len(weight_sets)], ds.tree_off, ds.parent, 1, Ns, ds.k_cache, ds.v_cache,
                                      ds.seq_stride, ds.head_stride, ds.ctx_len, L, ds.x, ds.out, ds.k_new, ds.v_new, None)
                ev.evict_accept_path(None, ds.tree_off, ds.parent, dt, tn, 1, pth, Ns, path_len, bonus)
            for i in range(10):
                step_s(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(60):
                step_s(i)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) * 1e6 / 60
            nsb = Us * expert_bytes + kv_bytes
            pts.append({"nodes": Ns, "us": round(us, 2), "union_experts": Us,
                        "hbm_frac_north_star": round(nsb / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                        "tokens_per_s": round(Ns / (us * 1e-6), 1)})
        out["sweep"] = pts

    # the same model at full depth: 48 layers + LM head + acceptance, tree sizes 8..128 at child noise 0.2 and 1.0,
    # ctx 4096 (`bench.py --stack` prints these as lines of their own, with the other stack workloads)
    if default_workload and not args.no_sweep:
        recs = []
        stack_bench(args, collect=recs)
        out["stack_48_layers_ctx4096"] = [{"nodes": r["nodes"], "sigma": r["sigma"], "ms": r["value"], "tokens_per_s": r["tokens_per_s"],
                                           "mean_union_per_layer": r["mean_union_per_layer"], "us_per_layer": r["us_per_layer"],
                                           "hbm_frac_north_star": r["hbm_frac_north_star"]} for r in recs]

    if not args.no_cpu:
        from oracle import evict_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        def oracle_step():
            orc.select_prefix(case["parent"], case["q"], cost, N)
            r = orc.verify_layer(cfg, case["W"], case["tree_off"], case["parent"], case["x"], case["K"], case["V"], case["ctx_len"])
            orc.accept_path(case["parent"], draft_tok, target_next)
            return r
        ref = oracle_step()  # (also warms the BLAS threads up)
        reps = 15  # about 7 s of CPU work at the default workload on all cores
        c0 = time.perf_counter()
        for _ in range(reps):
            oracle_step()
        c1 = time.perf_counter()
        one_thread_us, reps1 = None, 3
        try:
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):
                oracle_step()
                s0 = time.perf_counter()
                for _ in range(reps1):
                    oracle_step()
                one_thread_us = round((time.perf_counter() - s0) * 1e6 / reps1, 1)
        except Exception:
            one_thread_us = None
        rel = float(np.linalg.norm(res["out"] - ref["out"]) / np.linalg.norm(ref["out"]))
        out["cpu_baseline"] = {"value": round((c1 - c0) * 1e6 / reps, 1), "unit": "us", "cores": int(cores), "kind": "oracle",
                               "sample": f"{reps} full steps of the same workload on all host threads, mean (numpy float64 oracle: select + "
                                         f"layer + accept); single thread: {reps1} steps",
                               "single_thread_us": one_thread_us,
                               "gpu_vs_oracle_rel_l2": round(rel, 6)}
    print(json.dumps(out), flush=True)
    layer.close()


if __name__ == "__main__":
    main()
