"""Seeded random layer shapes, tree sizes, context lengths, batches and launch-shape knobs through the
whole layer protocol of test_gpu_layer.py (every stage against the CPU oracle): the kernels pick their
variants by shape, so the unusual combinations are where a variant boundary would show."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu

pytest.importorskip("paper_2605_00342_amd")
from test_gpu_layer import check_against_oracle, run_case  # noqa: E402


def random_case(seed):
    g = synth.philox(seed, 4242)
    dtype = "bf16" if g.random() < 0.7 else "f32"
    step = 32 if dtype == "bf16" else 16
    D = int(g.choice([64, 128]))
    Hkv = int(g.choice([1, 2, 4]))
    Hq = Hkv * int(g.choice([1, 2, 4, 8]))
    d = int(g.choice([256, 384, 512, 768, 1024]))
    E = int(g.choice([16, 32, 48, 64, 128, 256]))
    k = int(g.integers(1, min(8, E) + 1))
    F = step * int(g.integers(2, 13))
    n_shared = int(g.choice([0, 0, 1, 2]))
    cfg = synth.ModelCfg(f"rnd{seed}", dtype, d=d, Hq=Hq, Hkv=Hkv, D=D, E=E, k=k, F=F, n_shared=n_shared, theta=1e4,
                         router_norm="sigmoid" if g.random() < 0.3 else "softmax")
    batch = int(g.choice([1, 1, 1, 2, 3, 4]))
    n = int(g.choice([1, 2, 7, 16, 17, 31, 33, 64, 65, 100, 128]))
    if batch > 1:
        n = min(n, 48)
    Ls = [int(g.choice([0, 1, 5, 63, 64, 127, 128, 129, 300, 517])) for _ in range(batch)]
    tree = str(g.choice(["random", "eagle", "bfs", "chain", "star"]))
    sigma = float(g.choice([0.0, 0.1, 0.5, 1.0]))
    case = synth.make_case(cfg.name, n=n, L=Ls[0], seed=seed, sigma=sigma, tree=tree, batch=batch,
                           L_list=Ls if batch > 1 else None, cfg=cfg)
    tune = {}
    if g.random() < 0.5:
        tune["dense_kernel"] = int(g.choice([0, 1]))
        tune["dense_ntw"] = int(g.choice([0, 1, 2]))
    if g.random() < 0.5:
        tune["moe_gateup_kernel"] = int(g.choice([0, 1]))
    if g.random() < 0.3:
        tune["moe_nt"] = 2
    if g.random() < 0.3:
        tune["moe_down_kernel"] = 0
    if g.random() < 0.4:
        tune["attn_waves"] = int(g.choice([4, 8]))
        tune["attn_target_wgs"] = int(g.choice([2, 16, 512]))
    if g.random() < 0.4:  # (drawn last: the shapes of earlier seeds stay what they were)
        tune["moe_pair_down"] = int(g.choice([0, 1]))
        tune["moe_down_ws"] = int(g.choice([8, 16]))
    return cfg, case, tune, dict(n=n, Ls=Ls, tree=tree, sigma=sigma, batch=batch)


@pytest.mark.parametrize("seed", list(range(7000, 7048)))
def test_random_shape(seed):
    cfg, case, tune, what = random_case(seed)
    print(f"seed {seed}: {cfg} {what} tune={tune}", flush=True)
    info = check_against_oracle(case, run_case(case, tune=tune))
    assert cfg.k <= info["union"] <= min(cfg.E, case["x"].shape[0] * cfg.k)
