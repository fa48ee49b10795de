"""The allocation-free variant of acceptance under sampling (static device scratch inside the library)
gives exactly what evict_accept_path_sampled gives: two calls in a row through the C ABI, the second on
a smaller input, every output compared bit for bit; the size limit is an error, not a fault."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu

ev = pytest.importorskip("paper_2605_00342_amd")
from paper_2605_00342_amd import harness  # noqa: E402

DEV = "cuda:0"


def _case(seed, sizes, V):
    g = synth.philox(seed, 61)
    parents = [synth.tree_bfs_random(n, g) for n in sizes]
    tree_off, parent = synth.concat_trees(parents)
    T = int(tree_off[-1])
    logits = (3.0 * g.standard_normal((T, V))).astype(np.float32)
    tok = np.zeros(T, np.int32)
    for b, par in enumerate(parents):
        lo = int(tree_off[b])
        for u in range(len(par)):
            kids = [c for c in range(len(par)) if par[c] == u]
            top = np.argsort(-logits[lo + u])[: max(8, len(kids))]
            for c, t in zip(kids, g.permutation(top)[: len(kids)]):
                tok[lo + c] = t
    u_node = (g.random(T) ** 3).astype(np.float32)
    u_bonus = g.random(len(sizes)).astype(np.float32)
    return tree_off, parent, logits, tok, u_node, u_bonus


def _run(fn, ctx, c, V, temp, stride):
    tree_off, parent, logits, tok, u_node, u_bonus = c
    B, T = len(tree_off) - 1, int(tree_off[-1])
    i32 = torch.int32
    path = torch.full((B, stride), -7, dtype=i32, device=DEV)
    plen = torch.full((B,), -7, dtype=i32, device=DEV)
    bonus = torch.full((B,), -7, dtype=i32, device=DEV)
    fn(ctx, harness.dev_i32(tree_off), harness.dev_i32(parent), harness.dev_i32(tok), torch.from_numpy(logits).to(DEV), V, temp,
       torch.from_numpy(u_node).to(DEV), torch.from_numpy(u_bonus).to(DEV), B, T, path, stride, plen, bonus)
    torch.cuda.synchronize()
    return path.cpu().numpy(), plen.cpu().numpy(), bonus.cpu().numpy()


def test_noalloc_entry_point_equals_the_context_one_on_two_calls_in_a_row():
    cfg = synth.CONFIGS["tiny"]
    V = 640
    ctx = ev.evict_create(harness.model_desc(cfg), 256, 8, 16)
    big = _case(7, [40, 64, 9, 33, 1, 50], V)        # 197 nodes, 6 sequences
    small = _case(8, [12, 5], V)                     # 17 nodes: reuses the first rows of the static scratch
    for c, temp in ((big, 0.8), (small, 1.3)):
        ref = _run(ev.evict_accept_path_sampled, ctx, c, V, temp, 24)
        got = _run(ev.evict_accept_path_sampled_noalloc, None, c, V, temp, 24)
        for r, g_ in zip(ref, got):
            assert np.array_equal(r, g_)
        assert np.all(ref[1] >= 1)
    # with a context the status word is reported exactly as by the other entry point
    got = _run(ev.evict_accept_path_sampled_noalloc, ctx, small, V, 1.3, 24)
    assert np.array_equal(got[1], _run(ev.evict_accept_path_sampled, ctx, small, V, 1.3, 24)[1])
    assert ev.evict_device_status(ctx) == 0
    # beyond the static scratch: a clear error before anything is launched
    one = torch.zeros(8, dtype=torch.int32, device=DEV)
    onef = torch.zeros(8, device=DEV)
    with pytest.raises(ev.EvictError) as e:
        ev.evict_accept_path_sampled_noalloc(None, one, one, one, onef, 8, 1.0, onef, onef, 1, 4097, one, 4, one, one)
    assert e.value.code == 2 and "4096" in str(e.value)
    ev.evict_destroy(ctx)
