"""Host logic of the cost surface over (verification length, expert union): closed form of the
expected union (App. A) against the oracle's and a brute-force enumeration, recovery of a planted
surface, the collapse to C(k), and that a selection driven by the collapsed table equals the
oracle's on the same table."""
import itertools

import numpy as np
import pytest

from oracle import evict_oracle as orc

cm = pytest.importorskip("paper_2605_00342_amd.cost_model")


def test_expected_union_closed_form_against_oracle_and_enumeration():
    for E, k in [(16, 2), (128, 8), (256, 8), (64, 6)]:
        t = np.arange(0, 70)
        np.testing.assert_allclose(cm.expected_union(t, E, k), [orc.expected_unique_experts(E, k, int(v)) for v in t], rtol=1e-12)
    # brute force: 2 tokens, 4 experts, top-1 and top-2 sets drawn uniformly
    for E, k in [(4, 1), (4, 2), (5, 2)]:
        sets = list(itertools.combinations(range(E), k))
        mean = np.mean([len(set(a) | set(b)) for a in sets for b in sets])
        assert abs(cm.expected_union(2, E, k) - mean) < 1e-12
    assert cm.expected_union(0, 128, 8) == 0.0 and abs(cm.expected_union(1, 128, 8) - 8.0) < 1e-12


def test_planted_surface_is_recovered_and_collapsed():
    g = np.random.default_rng(5)
    k = np.tile(np.arange(1, 33), 2).astype(np.float64)
    u = np.concatenate([cm.expected_union(np.arange(1, 33), 128, 8) * 0.6, cm.expected_union(np.arange(1, 33), 128, 8)])
    ms = 0.08 + 0.0004 * k + 0.0011 * u
    coef, rms = cm.fit_cost_surface(k, u, ms)
    np.testing.assert_allclose(coef, [0.08, 0.0004, 0.0011], rtol=1e-9)
    assert rms < 1e-12
    coef_n, rms_n = cm.fit_cost_surface(k, u, ms * (1 + 0.01 * g.standard_normal(ms.size)))
    np.testing.assert_allclose(coef_n, coef, rtol=0.25)
    assert 0 < rms_n < 0.01
    # the surface evaluated at one point: the collapse with the union pinned to 40 at every length
    pinned = cm.collapse_cost(coef, 32, 128, 8, np.full(33, 40.0))
    assert pinned.shape == (33,) and abs(pinned[7] - (0.08 + 0.0004 * 7 + 0.0011 * 40)) < 1e-6
    # closed-form unions, then measured ones for the lengths that have them
    c0 = cm.collapse_cost(coef, 32, 128, 8)
    want = 0.08 + 0.0004 * np.arange(33) + 0.0011 * cm.expected_union(np.arange(33), 128, 8)
    np.testing.assert_allclose(c0[1:], want[1:], rtol=1e-6)
    assert c0[0] == c0[1]
    meas = np.zeros(33); meas[1:17] = np.arange(1, 17) * 3.0
    c1 = cm.collapse_cost(coef, 32, 128, 8, meas)
    np.testing.assert_allclose(c1[5], 0.08 + 0.0004 * 5 + 0.0011 * 15.0, rtol=1e-6)
    np.testing.assert_allclose(c1[20], want[20], rtol=1e-6)
    assert np.all(np.diff(c0[1:]) > 0)  # more nodes and more experts never cost less on this surface


def test_degenerate_fits_are_refused():
    with pytest.raises(ValueError):
        cm.fit_cost_surface([1, 2], [8, 15], [0.1, 0.2])
    with pytest.raises(ValueError):  # U an exact linear function of k: the two axes cannot be told apart
        cm.fit_cost_surface([1, 2, 3, 4], [8, 16, 24, 32], [0.1, 0.2, 0.3, 0.4])
    with pytest.raises(ValueError):
        cm.collapse_cost(np.array([-1.0, 0.0, 0.0]), 8, 16, 2)


def test_collapsed_table_makes_selection_stop_earlier_when_experts_cost_more():
    import synth
    case = synth.make_case("tiny", n=8, L=64, seed=0)
    cheap = cm.collapse_cost(np.array([1.0, 0.0, 0.001]), 8, 16, 2)
    dear = cm.collapse_cost(np.array([0.05, 0.0, 0.2]), 8, 16, 2)
    k_cheap = orc.select_prefix(case["parent"], case["q"], cheap, 8)["k_star"]
    k_dear = orc.select_prefix(case["parent"], case["q"], dear, 8)["k_star"]
    assert 1 <= k_dear <= k_cheap <= 8


def test_cost_table_file_round_trip_and_refusals(tmp_path):
    cost = cm.collapse_cost(np.array([0.08, 0.0004, 0.0011]), 64, 128, 8)
    path = str(tmp_path / "cost.txt")
    key = cm.table_key("gfx950", "qwen3-30b-a3b", "bf16", 48, 2048)
    cm.save_cost_table(path, cost, key)
    back = cm.load_cost_table(path, key)
    assert back.dtype == np.float32 and np.array_equal(back, cost)  # 9 significant digits: bit-exact floats
    assert np.array_equal(cm.load_cost_table(path), cost)           # any key
    head = open(path).read().splitlines()[0]
    assert head == "evict-cost-table 1 64 gfx950:qwen3-30b-a3b:bf16:L48:ctx2048"
    with pytest.raises(ValueError):  # profiled for another context length
        cm.load_cost_table(path, cm.table_key("gfx950", "qwen3-30b-a3b", "bf16", 48, 8192))
    with pytest.raises(ValueError):
        cm.save_cost_table(path, cost, "two words")
    with pytest.raises(ValueError):
        cm.save_cost_table(path, [0.1, -1.0], key)
    with pytest.raises(ValueError):
        cm.load_cost_table(str(tmp_path / "absent.txt"))
    bad = tmp_path / "bad.txt"
    bad.write_text("evict-cost-table 1 2 k\n0.1\n-0.2\n0.3\n")  # a cost must be positive (Eq. 10 divides by it)
    with pytest.raises(ValueError):
        cm.load_cost_table(str(bad))
    short = tmp_path / "short.txt"
    short.write_text("evict-cost-table 1 3 k\n0.1\n0.2\n")
    with pytest.raises(ValueError):
        cm.load_cost_table(str(short))
    other = tmp_path / "other.txt"
    other.write_text("something else\n")
    with pytest.raises(ValueError):
        cm.load_cost_table(str(other))


def test_fit_is_pinned_to_numpy_least_squares():
    # the library's centred normal equations against a library least-squares solve on random points
    g = np.random.default_rng(11)
    k = g.integers(1, 129, 200).astype(np.float64)
    u = 128 * (1 - (1 - 8 / 128) ** k) * g.uniform(0.5, 1.0, 200)
    ms = 0.07 + 0.0005 * k + 0.0012 * u + 0.002 * g.standard_normal(200)
    coef, rms = cm.fit_cost_surface(k, u, ms)
    A = np.stack([np.ones_like(k), k, u], axis=1)
    want, *_ = np.linalg.lstsq(A, ms, rcond=None)
    np.testing.assert_allclose(coef, want, rtol=1e-8)
    assert abs(rms - np.sqrt(np.mean((A @ want - ms) ** 2))) < 1e-12
