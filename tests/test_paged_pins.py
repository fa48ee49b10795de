"""Pins of the paged-cache reading / commit used as the reference for the paged entry points: a
storage layout, so the pins are round trips against the contiguous definitions (themselves pinned
in test_oracle_pins.py) and hand-placed rows."""
import numpy as np
import pytest

import synth
from oracle import evict_oracle as orc


@pytest.mark.parametrize("P,Ls", [(1, [5]), (4, [9, 0, 16]), (16, [33, 7]), (64, [40])])
def test_view_of_scattered_pages_is_the_contiguous_cache(P, Ls):
    cfg = synth.CONFIGS["tiny"]
    g = synth.philox(3, P)
    kv = [synth.kv_cache(cfg, L, g) for L in Ls]
    Ks, Vs = [k for k, _ in kv], [v for _, v in kv]
    pk, pv, table, n_pages = synth.to_pages(Ks, Vs, P, [L + 6 for L in Ls], g)
    assert pk.shape == (n_pages, cfg.Hkv, P, cfg.D)
    used = table[table < n_pages]
    assert len(set(used.tolist())) == used.size                      # no page serves two places
    for b, L in enumerate(Ls):
        assert np.array_equal(orc.paged_view(pk, table[b], L, P), Ks[b])
        assert np.array_equal(orc.paged_view(pv, table[b], L, P), Vs[b])


def test_hand_placed_rows():
    # 3 pages of 2 positions, one head, D = 1; sequence uses pages 2 then 0
    pool = np.array([[[[10.], [11.]]], [[[20.], [21.]]], [[[30.], [31.]]]])
    assert orc.paged_view(pool, [2, 0], 3, 2)[0, :, 0].tolist() == [30., 31., 10.]
    pk, pv = pool.copy(), pool.copy()
    k_new = np.array([[[1.]], [[2.]], [[3.]]]); v_new = -k_new
    L = orc.kv_commit_paged(pk, pv, [2, 0], 1, k_new, v_new, [0, 2], 2)   # positions 1 and 2
    assert L == 3
    assert pk[2, 0, 1, 0] == 1. and pk[0, 0, 0, 0] == 3. and pv[0, 0, 0, 0] == -3.
    assert pk[2, 0, 0, 0] == 30. and pk[0, 0, 1, 0] == 11. and np.array_equal(pk[1], pool[1])   # nothing else moved


@pytest.mark.parametrize("P", [1, 4, 16])
def test_paged_commit_equals_contiguous_commit(P):
    cfg = synth.CONFIGS["tiny"]
    g = synth.philox(9, P)
    L, n = 13, 8
    K, V = synth.kv_cache(cfg, L, g)
    k_new = g.standard_normal((n, cfg.Hkv, cfg.D)).astype(np.float32)
    v_new = g.standard_normal((n, cfg.Hkv, cfg.D)).astype(np.float32)
    path = [0, 2, 5, 6]
    pk, pv, table, _ = synth.to_pages([K], [V], P, [L + n], g)
    K2, V2 = orc.kv_commit(K, V, k_new, v_new, path)
    L2 = orc.kv_commit_paged(pk, pv, table[0], L, k_new, v_new, path, P)
    assert L2 == L + len(path)
    assert np.array_equal(orc.paged_view(pk, table[0], L2, P), K2)
    assert np.array_equal(orc.paged_view(pv, table[0], L2, P), V2)
