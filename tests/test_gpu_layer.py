"""GPU parity of evict_verify_layer against the CPU oracle on seeded synthetic cases.

Routing indices and the expert union are compared bit-exactly, stage-wise: the oracle's router
is run on the normalised hidden state the GPU handed to its own router (tokens whose k-th
and (k+1)-th scores differ by < 1e-4 are excluded and counted). Hidden outputs are compared
end to end within 1e-4 (fp32) / 2e-2 (bf16) relative L2."""
import numpy as np
import pytest
import torch

import synth
from oracle import evict_oracle as orc

pytestmark = pytest.mark.gpu

ev = pytest.importorskip("paper_2605_00342_amd")
from paper_2605_00342_amd import harness  # noqa: E402

TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_l2(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-30))


def row_rel_l2_max(a, b):
    """Largest relative L2 error of any single token row: one wrong token in a large call cannot hide in it."""
    a = np.asarray(a, np.float64).reshape(len(a), -1)
    b = np.asarray(b, np.float64).reshape(len(b), -1)
    return float(np.max(np.linalg.norm(a - b, axis=1) / np.maximum(np.linalg.norm(b, axis=1), 1e-30)))


ROW_FACTOR = 3.0  # per-row bound = ROW_FACTOR x the whole-tensor tolerance


def run_case(case, max_tokens=None, tune=None):
    cfg = case["cfg"]
    T = int(case["tree_off"][-1])
    layer = harness.DeviceLayer(cfg, case["W"], max_tokens or T, len(case["ctx_len"]), int(max(case["ctx_len"])))
    for key, value in (tune or {}).items():
        ev.evict_tune(layer.ctx, key, value)
    dc = harness.DeviceCase(case)
    dc.run(layer)
    got = dc.results()
    assert ev.evict_device_status(layer.ctx) == 0
    layer.close()
    return got


def check_against_oracle(case, got):
    cfg = case["cfg"]
    tol = TOL[cfg.dtype]
    ref = orc.verify_layer(cfg, case["W"], case["tree_off"], case["parent"], case["x"], case["K"], case["V"],
                           case["ctx_len"])
    T = case["x"].shape[0]
    # --- attention part, end to end
    assert rel_l2(got["q"], ref["q"]) < tol, "q"
    assert rel_l2(got["k_new"], ref["k_new"]) < tol, "k_new"
    assert rel_l2(got["v_new"], ref["v_new"]) < tol, "v_new"
    assert rel_l2(got["attn_out"], ref["o"]) < tol, "attention output"
    assert rel_l2(got["h"], ref["h"]) < tol, "h"
    assert rel_l2(got["h_norm"], ref["h_norm"]) < tol, "h_norm"
    # no single token row may be far off either
    for name, g_, r_ in (("q", got["q"], ref["q"]), ("attention output", got["attn_out"], ref["o"]), ("h", got["h"], ref["h"])):
        worst = row_rel_l2_max(g_, r_)
        assert worst < ROW_FACTOR * tol, f"{name}: worst token row {worst}"
    # --- router, stage-wise on the GPU's own normalised hidden state: bit-exact indices
    idx, w, logits = orc.router_topk(got["h_norm"], case["W"]["wg"], cfg.k, cfg.router_norm)
    np.testing.assert_allclose(got["router_logits"], logits, rtol=0, atol=2e-5)
    margin = orc.router_margin(logits, cfg.k)
    # ordering inside the top-k can also flip on near-equal neighbours; find the tightest gap
    srt = -np.sort(-logits.astype(np.float64), axis=-1)[:, :cfg.k + 1]
    tight = np.min(srt[:, :-1] - srt[:, 1:], axis=-1) if cfg.E > cfg.k else np.min(srt[:, :-1] - srt[:, 1:], axis=-1)
    keep = tight >= 1e-4
    excluded = int((~keep).sum())
    assert excluded <= max(2, T // 8), f"{excluded} near-tie tokens"
    assert np.array_equal(got["topk_idx"][keep], idx[keep])
    np.testing.assert_allclose(got["topk_w"][keep], w[keep], rtol=0, atol=2e-6)
    assert np.all(margin[keep] >= 1e-4)
    # --- union of the GPU's routing, bit-exact
    un = orc.expert_union(got["topk_idx"], cfg.E)
    assert got["union_count"] == un["union_count"]
    assert np.array_equal(got["union_ids"][:un["union_count"]], un["union_ids"])
    assert np.all(got["union_ids"][un["union_count"]:] == -1)
    assert np.array_equal(got["hist"], un["hist"])
    assert cfg.k <= got["union_count"] <= min(cfg.E, T * cfg.k)
    # --- MoE stage-wise: oracle experts + combine on the GPU's h / h_norm / routing
    y = orc.moe_experts(np.asarray(got["h_norm"], np.float64), got["topk_idx"], case["W"], cfg.dtype)
    shared = None
    if cfg.n_shared:
        shared = sum(orc.expert_mlp(np.asarray(got["h_norm"], np.float64), case["W"]["ws_gate"][s], case["W"]["ws_up"][s],
                                    case["W"]["ws_down"][s], cfg.dtype) for s in range(cfg.n_shared))
    out_stage = orc.moe_combine(got["h"], y, got["topk_w"], shared)
    out_stored = orc.handoff(out_stage, cfg.dtype)     # the layer output is stored in the storage type
    assert rel_l2(got["out"], out_stored) < (1e-3 if cfg.dtype == "bf16" else 1e-5), "MoE stage"
    worst = row_rel_l2_max(got["out"], out_stored)
    assert worst < ROW_FACTOR * (1e-3 if cfg.dtype == "bf16" else 1e-5), f"MoE stage: worst token row {worst}"
    # error measured against the size of the MoE contribution itself (a wrong expert sum gives ~1)
    moe_part = np.linalg.norm(got["out"] - out_stored) / np.linalg.norm(out_stage - np.asarray(got["h"], np.float64))
    assert moe_part < (5e-2 if cfg.dtype == "bf16" else 1e-4), f"MoE contribution {moe_part}"
    # --- hidden output end to end
    flips = int((np.sort(got["topk_idx"], -1) != np.sort(ref["topk_idx"], -1)).any(-1).sum())
    err = rel_l2(got["out"], ref["out"])
    assert err < tol, f"out rel-L2 {err} (routing flips vs end-to-end oracle: {flips})"
    # per token row, on the rows whose routing agrees with the end-to-end oracle's (a flipped near-tie swaps an expert)
    same = ~(np.sort(got["topk_idx"], -1) != np.sort(ref["topk_idx"], -1)).any(-1)
    if same.any():
        worst = row_rel_l2_max(got["out"][same], ref["out"][same])
        assert worst < ROW_FACTOR * tol, f"out: worst token row {worst}"
    return {"err": err, "flips": flips, "excluded": excluded, "union": got["union_count"]}


def test_tiny_fp32_config_seed0():
    case = synth.make_case("tiny", n=8, L=64, seed=0)
    info = check_against_oracle(case, run_case(case))
    assert info["flips"] == 0


@pytest.mark.parametrize("n,L,tree,seed", [(1, 64, "random", 1), (8, 0, "random", 2), (13, 37, "random", 3),
                                           (33, 130, "eagle", 4), (128, 70, "bfs", 5), (70, 65, "chain", 6)])
def test_tiny_fp32_shapes(n, L, tree, seed):
    case = synth.make_case("tiny", n=n, L=L, seed=seed, tree=tree)
    check_against_oracle(case, run_case(case))


@pytest.mark.parametrize("n,L,tree,seed", [(8, 64, "random", 10), (19, 100, "eagle", 11), (40, 257, "bfs", 12),
                                           (1, 5, "random", 13), (128, 64, "eagle", 14)])
def test_mini_bf16_shapes(n, L, tree, seed):
    case = synth.make_case("mini_bf16", n=n, L=L, seed=seed, tree=tree)
    check_against_oracle(case, run_case(case))


@pytest.mark.parametrize("n,L,tree,seed", [(8, 64, "random", 20), (33, 150, "eagle", 21), (70, 129, "bfs", 22)])
def test_sigmoid_router_256_experts_64_wide_heads(n, L, tree, seed):
    """Sigmoid-normalised router weights (Sec. 2.2), 256 experts / 8 active, head dimension 64."""
    case = synth.make_case("mini_sigmoid", n=n, L=L, seed=seed, tree=tree)
    check_against_oracle(case, run_case(case))


@pytest.mark.parametrize("cfg_name,n,L,tree,seed,batch", [
    ("mini_bf16", 128, 700, "eagle", 30, 1),      # 32 row tiles, 6 chunks with a ragged last one
    ("mini_bf16", 40, 1, "bfs", 31, 1),           # a single cache key
    ("mini_sigmoid", 70, 300, "bfs", 32, 1),      # 64-wide heads
    ("mini_bf16", 50, 260, "bfs", 33, 3),         # batch with different context lengths
])
def test_attention_variants_agree_with_oracle(cfg_name, n, L, tree, seed, batch):
    """Both workgroup shapes of the bf16 attention kernel (4 wavefronts / one LDS buffer, 8 wavefronts /
    two buffers with the next chunk in flight) and small split targets, forced through evict_tune."""
    L_list = [L, max(1, L // 3), L // 2 + 7][:batch] if batch > 1 else None
    case = synth.make_case(cfg_name, n=n, L=L, seed=seed, tree=tree, batch=batch, L_list=L_list)
    for tune in ({"attn_waves": 8}, {"attn_waves": 8, "attn_target_wgs": 4}, {"attn_waves": 4, "attn_target_wgs": 2}):
        check_against_oracle(case, run_case(case, tune=tune))


def test_batched_trees_fp32_and_bf16():
    for name, seed in (("tiny", 20), ("mini_bf16", 21)):
        case = synth.make_case(name, n=12, L=0, seed=seed, tree="bfs", batch=3, L_list=[70, 5, 129])
        check_against_oracle(case, run_case(case))


def test_shared_experts_and_mha():
    cfg = synth.ModelCfg("t_shared", "bf16", d=256, Hq=4, Hkv=4, D=64, E=16, k=3, F=96, n_shared=2, theta=1e4)
    case = synth.make_case("t_shared", n=24, L=50, seed=30, tree="bfs", cfg=cfg)
    check_against_oracle(case, run_case(case))


def test_all_tokens_to_one_expert_spans_token_tiles():
    # identical hidden states: every token picks the same k experts (union == k), so each expert
    # sees all 40 tokens: several 16-token tiles with a ragged tail
    case = synth.make_case("mini_bf16", n=40, L=16, seed=31, tree="star", sigma=0.0)
    got = run_case(case)
    assert got["union_count"] == case["cfg"].k
    check_against_oracle(case, got)


def test_two_tile_work_list_slots():
    """Grouped GEMMs with 32-token work-list slots (two 16-token tiles per workgroup), forced through evict_tune:
    experts with 1..3 slots and ragged tails, shared experts, fp32 and bf16, both down-projection kernels."""
    cases = [synth.make_case("mini_bf16", n=40, L=16, seed=31, tree="star", sigma=0.0),      # 40 tokens per expert
             synth.make_case("mini_bf16", n=128, L=64, seed=14, tree="eagle"),
             synth.make_case("tiny", n=70, L=20, seed=34, tree="bfs"),
             synth.make_case("mini_sigmoid", n=90, L=33, seed=35, tree="bfs")]
    cfg = synth.ModelCfg("t_shared", "bf16", d=256, Hq=4, Hkv=4, D=64, E=16, k=3, F=96, n_shared=2, theta=1e4)
    cases.append(synth.make_case("t_shared", n=50, L=50, seed=36, tree="bfs", cfg=cfg))
    for case in cases:
        check_against_oracle(case, run_case(case, tune={"moe_nt": 2}))
        check_against_oracle(case, run_case(case, tune={"moe_nt": 2, "moe_down_kernel": 0}))
    # full-size layer, tightly correlated tokens (experts with 17..64 tokens): the strip-pair gate/up kernel with
    # two token tiles per slot
    case = synth.make_case("qwen3", n=64, L=200, seed=38, sigma=0.1)
    got = run_case(case, tune={"moe_nt": 2, "moe_gateup_kernel": 1})
    assert got["hist"].max() > 16
    check_against_oracle(case, got)


def test_down_projection_paired_slots_and_16_strip_workgroups():
    """The down projection taking two consecutive 16-token slots of an expert through one weight stream, and its
    workgroups of 16 strips, forced through evict_tune on small shapes: experts with 1..3 slots and ragged tails
    (odd slot counts leave a last slot unpaired), shared experts, fp32 and bf16; the paired result is bit-identical
    to the unpaired one (same products, same order per output)."""
    cases = [synth.make_case("mini_bf16", n=40, L=16, seed=31, tree="star", sigma=0.0),      # 40 tokens per expert: 3 slots
             synth.make_case("mini_bf16", n=128, L=64, seed=14, tree="eagle"),
             synth.make_case("tiny", n=70, L=20, seed=34, tree="bfs"),
             synth.make_case("mini_sigmoid", n=90, L=33, seed=35, tree="bfs")]
    cfg = synth.ModelCfg("t_shared", "bf16", d=256, Hq=4, Hkv=4, D=64, E=16, k=3, F=96, n_shared=2, theta=1e4)
    cases.append(synth.make_case("t_shared", n=50, L=50, seed=36, tree="bfs", cfg=cfg))
    for case in cases:
        plain = run_case(case, tune={"moe_pair_down": 0, "moe_down_ws": 8})
        paired = run_case(case, tune={"moe_pair_down": 1, "moe_down_ws": 8})
        check_against_oracle(case, paired)
        assert np.array_equal(paired["out"], plain["out"])
    # full-size layer (the 16-strip variant is built for its expert width): many tokens per expert
    case = synth.make_case("qwen3", n=128, L=100, seed=39, sigma=0.2)
    base = run_case(case, tune={"moe_pair_down": 0, "moe_down_ws": 8})
    assert base["hist"].max() > 32
    for tune in ({"moe_pair_down": 1, "moe_down_ws": 16}, {"moe_pair_down": 0, "moe_down_ws": 16}, {"moe_pair_down": 1, "moe_down_ws": 8}):
        got = run_case(case, tune=tune)
        check_against_oracle(case, got)
        assert np.array_equal(got["out"], base["out"])
    # expert width 1408 (44 contraction blocks): the 16-strip variant alone and with paired slots (88 KiB operand),
    # shared experts with 8 slots each
    case = synth.make_case("dsv2lite", n=128, L=64, seed=40, sigma=0.2)
    base = run_case(case, tune={"moe_pair_down": 0, "moe_down_ws": 8})
    check_against_oracle(case, base)
    for tune in ({"moe_pair_down": 1, "moe_down_ws": 16}, {"moe_pair_down": 0, "moe_down_ws": 16}):
        assert np.array_equal(run_case(case, tune=tune)["out"], base["out"])


def test_gateup_one_strip_pair_per_wavefront():
    """The second gate/up decomposition (token operand in LDS, one strip pair per wavefront), forced through
    evict_tune: multi-tile experts, shared experts, fp32 and bf16, 256 experts, and the full-size layer."""
    cases = [synth.make_case("mini_bf16", n=40, L=16, seed=31, tree="star", sigma=0.0),
             synth.make_case("mini_bf16", n=128, L=64, seed=14, tree="eagle"),
             synth.make_case("tiny", n=70, L=20, seed=34, tree="bfs"),
             synth.make_case("mini_sigmoid", n=90, L=33, seed=35, tree="bfs"),
             synth.make_case("qwen3", n=32, L=300, seed=37)]
    cfg = synth.ModelCfg("t_shared", "bf16", d=256, Hq=4, Hkv=4, D=64, E=16, k=3, F=128, n_shared=2, theta=1e4)
    cases.append(synth.make_case("t_shared", n=50, L=50, seed=36, tree="bfs", cfg=cfg))
    for case in cases:
        check_against_oracle(case, run_case(case, tune={"moe_gateup_kernel": 1}))
    # token operand staged with direct global-to-LDS loads (full-size shape only: 64 contraction blocks), single
    # and several token tiles per expert, and bit-identical to the register-staged variant
    for case in (cases[4], synth.make_case("qwen3", n=128, L=100, seed=39, sigma=0.2)):
        got = run_case(case, tune={"moe_gateup_kernel": 1, "moe_lds_dma": 1})
        check_against_oracle(case, got)
        assert np.array_equal(got["out"], run_case(case, tune={"moe_gateup_kernel": 1, "moe_lds_dma": 0})["out"])
        # few workgroups, so each takes many chunks in turn and restages its operand in between
        few = run_case(case, tune={"moe_gateup_kernel": 1, "moe_lds_dma": 1, "moe_grid": 40})
        assert np.array_equal(got["out"], few["out"])


def test_chain_tree_equals_token_by_token_decode_on_gpu():
    # verifying a chain of n nodes equals n single-node verifications with a growing cache
    case = synth.make_case("tiny", n=5, L=30, seed=32, tree="chain")
    cfg = case["cfg"]
    full = run_case(case)
    K = case["K"][0].copy(); V = case["V"][0].copy()
    for i in range(5):
        single = dict(case)
        single.update(tree_off=np.array([0, 1], np.int32), parent=np.array([-1], np.int32), parents=[np.array([-1], np.int32)],
                      x=case["x"][i:i + 1], K=[K], V=[V], ctx_len=np.array([30 + i], np.int32))
        r = run_case(single)
        assert rel_l2(r["out"], full["out"][i:i + 1]) < 1e-5
        K = np.concatenate([K, np.transpose(r["k_new"], (1, 0, 2))], axis=1)
        V = np.concatenate([V, np.transpose(r["v_new"], (1, 0, 2))], axis=1)


def test_deterministic_bitwise():
    case = synth.make_case("mini_bf16", n=32, L=100, seed=33, tree="eagle")
    a, b = run_case(case), run_case(case)
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["topk_idx"], b["topk_idx"])


def test_qwen3_shaped_layer_n32_full_size():
    case = synth.make_case("qwen3", n=32, L=2048, seed=1000)
    got = run_case(case)
    info = check_against_oracle(case, got)
    print("qwen3 N=32:", info)


def test_batched_qwen3_shaped_full_size_four_trees():
    # configs[4] shape for one layer: 4 sequences, N = 64 each, contexts between 2048 and 8192
    case = synth.make_case("qwen3", n=64, L=0, seed=1004, batch=4, L_list=[2048, 8192, 5000, 3333], tree="bfs")
    got = run_case(case)
    info = check_against_oracle(case, got)
    print("qwen3 4 x N=64:", info)


def test_dsv2lite_shaped_layer_full_size():
    # configs[3] layer shape: MHA 16 x 128, 64 experts top-6 + 2 shared, d_ff 1408, ctx 8192, N = 64
    case = synth.make_case("dsv2lite", n=64, L=8192, seed=1003)
    got = run_case(case)
    info = check_against_oracle(case, got)
    print("dsv2lite N=64:", info)


@pytest.mark.parametrize("cfg_name,seed", [("qwen3_235b_tp8", 1005), ("ling_flash2_tp4", 1006)])
def test_tensor_parallel_share_of_the_larger_targets_full_size(cfg_name, seed):
    # one GPU's share of the 128-expert / TP=8 and 256-expert / TP=4 targets (App. C.2), N = 32, ctx 2048
    case = synth.make_case(cfg_name, n=32, L=2048, seed=seed)
    got = run_case(case)
    info = check_against_oracle(case, got)
    print(cfg_name, "N=32:", info)


@pytest.mark.parametrize("n,sigma,seed", [(128, 1.0, 1010), (8, 0.2, 1011)])
def test_qwen3_shaped_layer_sweep_extremes_full_size(n, sigma, seed):
    # configs[2]: the two ends of the tree-size / child-noise sweep at ctx 4096, default launch configuration
    # (N = 128 takes the strip-pair-per-wavefront gate/up kernel and 8-wavefront attention workgroups)
    case = synth.make_case("qwen3", n=n, L=4096, seed=seed, sigma=sigma)
    got = run_case(case)
    info = check_against_oracle(case, got)
    print(f"qwen3 N={n} sigma={sigma}:", info)


def test_dense_projections_one_strip_per_wavefront():
    """The many-token decomposition of the QKV / output projections (token operand in LDS, one strip per
    wavefront), forced through evict_tune on small and ragged token counts, both workgroup shapes, fp32 and
    bf16, a strip count that is not a multiple of the strips per workgroup (t_odd: 28 QKV strips; its output
    projection has a contraction length the kernel does not take and stays on the other one), a batch, and
    the full-size layer."""
    cfg_odd = synth.ModelCfg("t_odd", "bf16", d=512, Hq=5, Hkv=1, D=64, E=16, k=2, F=64, theta=1e4)
    cases = [synth.make_case("mini_bf16", n=40, L=16, seed=61, tree="bfs"),
             synth.make_case("tiny", n=13, L=37, seed=62),
             synth.make_case("mini_sigmoid", n=33, L=50, seed=63),
             synth.make_case("t_odd", n=21, L=30, seed=64, tree="bfs", cfg=cfg_odd),
             synth.make_case("mini_bf16", n=50, L=60, seed=65, tree="bfs", batch=3, L_list=[60, 5, 33])]
    for case in cases:
        for tune in ({"dense_kernel": 1, "dense_ntw": 2}, {"dense_kernel": 1, "dense_ntw": 1}):
            check_against_oracle(case, run_case(case, tune=tune))
    case = synth.make_case("qwen3", n=32, L=300, seed=66)
    check_against_oracle(case, run_case(case, tune={"dense_kernel": 1}))
    # and the default choice equals the contraction-split kernels within rounding on a many-token call
    case = synth.make_case("mini_bf16", n=128, L=64, seed=14, tree="eagle")
    a, b = run_case(case), run_case(case, tune={"dense_kernel": 0})
    assert rel_l2(a["q"], b["q"]) < 1e-2 and rel_l2(a["h"], b["h"]) < 1e-2


@pytest.mark.parametrize("E,k,n,seed", [(512, 8, 40, 81), (1024, 6, 70, 82), (320, 3, 9, 83)])
def test_more_than_256_experts(E, k, n, seed):
    """Above 256 experts TopK keeps its keys in LDS instead of registers (and TopK / union are two launches)."""
    cfg = synth.ModelCfg(f"many{E}", "bf16", d=256, Hq=4, Hkv=2, D=64, E=E, k=k, F=64, theta=1e4)
    case = synth.make_case(cfg.name, n=n, L=50, seed=seed, tree="bfs", cfg=cfg)
    check_against_oracle(case, run_case(case))


@pytest.mark.parametrize("cfg_name", ["mini_bf16", "mini_sigmoid"])
def test_largest_call_eight_trees_of_128_nodes(cfg_name):
    """1024 tokens in one call (8 trees of the largest size); with 8 active experts that is the limit of
    8192 token-expert pairs, where the grouping leaves the bitmask path (masks no longer fit in LDS)."""
    case = synth.make_case(cfg_name, n=128, L=40, seed=91, tree="bfs", batch=8, L_list=[40, 0, 129, 7, 300, 64, 1, 200])
    info = check_against_oracle(case, run_case(case))
    print(cfg_name, "8 x 128:", info)


@pytest.mark.parametrize("cfg_name,n,L,seed", [("mini_bf16", 8, 12000, 95), ("tiny", 5, 12100, 96), ("mini_bf16", 40, 9999, 97),
                                               ("mini_bf16", 8, 100000, 99), ("mini_sigmoid", 16, 40000, 100)])
def test_longest_contexts(cfg_name, n, L, seed):
    """Long contexts: close to the fp32 limit of 12160 positions, and 40k / 100k positions with bf16 storage
    (rotary angles at such positions are formed in double on the device)."""
    case = synth.make_case(cfg_name, n=n, L=L, seed=seed)
    check_against_oracle(case, run_case(case))


def test_context_limit_is_an_error_not_a_fault():
    case = synth.make_case("tiny", n=4, L=8, seed=98)
    with pytest.raises(ev.EvictError):
        harness.DeviceLayer(case["cfg"], case["W"], 4, 1, 20000)
    with pytest.raises(ev.EvictError):          # more than 8192 token-expert pairs
        harness.DeviceLayer(case["cfg"], case["W"], 5000, 1, 64)
