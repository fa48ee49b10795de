"""Pins of the oracle's acceptance rule under sampling (Sec. 2.1, Eq. 3) against things fixed
outside it: hand-computed thresholds, the greedy rule as its one-hot limit, and the property
the paper states for it -- the emitted tokens follow the target distribution -- by simulation,
with planted mistakes shown to break that property."""
import numpy as np
import pytest

import synth
from oracle import evict_oracle as orc


def test_thresholds_worked_by_hand():
    # root with two children carrying tokens 0 and 1; target at the root p = (0.5, 0.3, 0.2)
    parent = np.array([-1, 0, 0], np.int32)
    tok = np.array([9, 0, 1], np.int32)
    P = np.array([[0.5, 0.3, 0.2], [1.0, 0.0, 0.0], [0.0, 0.0, 1.0]])
    # first child accepted iff u1 < 0.5
    path, bonus = orc.accept_path_sampled(parent, tok, P, [0, 0.49, 0.0], 0.0)
    assert list(path) == [0, 1] and bonus == 0            # then a draw from P[1] = token 0
    # rejected; second child sees 0.3 / (1 - 0.5) = 0.6
    path, bonus = orc.accept_path_sampled(parent, tok, P, [0, 0.6, 0.59], 0.7)
    assert list(path) == [0, 2] and bonus == 2
    path, bonus = orc.accept_path_sampled(parent, tok, P, [0, 0.6, 0.61], 0.7)
    assert list(path) == [0] and bonus == 2               # residual is all on token 2
    # residual after one rejection only (single child): (0, 0.6, 0.4)
    parent1, tok1 = np.array([-1, 0], np.int32), np.array([9, 0], np.int32)
    assert orc.accept_path_sampled(parent1, tok1, P[:2], [0, 0.5], 0.59)[1] == 1
    assert orc.accept_path_sampled(parent1, tok1, P[:2], [0, 0.5], 0.60)[1] == 2
    # trace carries the probabilities that were used
    _, _, trace, cdf = orc.accept_path_sampled(parent, tok, P, [0, 0.6, 0.61], 0.7, with_trace=True)
    assert [c for c, _, _ in trace] == [1, 2] and np.allclose([p for _, p, _ in trace], [0.5, 0.6])
    assert np.allclose(cdf, [0, 0, 1])


def test_repeated_sibling_token_cannot_be_accepted_twice():
    parent = np.array([-1, 0, 0], np.int32)
    tok = np.array([9, 1, 1], np.int32)
    P = np.array([[0.2, 0.8], [0.5, 0.5], [0.5, 0.5]])
    path, bonus = orc.accept_path_sampled(parent, tok, P, [0, 0.9, 0.0], 0.3)
    assert list(path) == [0] and bonus == 0  # second sibling has probability 0 after the removal


@pytest.mark.parametrize("seed", range(6))
def test_one_hot_target_is_the_greedy_rule(seed):
    g = synth.philox(seed, 41)
    n, V = 40, 17
    parent = synth.tree_random_parents(n, 6, g)
    nxt = g.integers(0, V, n).astype(np.int32)
    tok = synth.plant_draft_tokens(parent, nxt, V, g)
    P = np.zeros((n, V))
    P[np.arange(n), nxt] = 1.0
    path, bonus = orc.accept_path_sampled(parent, tok, P, g.random(n), g.random())
    rp, rb = orc.accept_path(parent, tok, nxt)
    assert list(path) == list(rp) and bonus == rb


def _simulate(fn, parent, tok, P, trials, seed):
    g = np.random.Generator(np.random.Philox(seed))
    V = P.shape[1]
    first = np.zeros(V)
    second = {}
    for _ in range(trials):
        path, bonus = fn(parent, tok, P, g.random(len(parent)), g.random())
        emitted = [int(tok[c]) for c in path[1:]] + [int(bonus)]
        first[emitted[0]] += 1
        if len(emitted) > 1:
            second.setdefault(int(path[1]), np.zeros(V))[emitted[1]] += 1
    return first / trials, second


TREE_PARENT = np.array([-1, 0, 0, 0, 1, 1, 2], np.int32)
TREE_TOK = np.array([0, 2, 4, 1, 3, 0, 5], np.int32)


def _target(seed, n, V):
    g = synth.philox(seed, 42)
    P = g.random((n, V)) ** 2 + 0.02
    return P / P.sum(axis=1, keepdims=True)


def test_emitted_tokens_follow_the_target_distribution():
    P = _target(1, len(TREE_PARENT), 6)
    trials = 40000
    first, second = _simulate(orc.accept_path_sampled, TREE_PARENT, TREE_TOK, P, trials, 7)
    sd = np.sqrt(P[0] * (1 - P[0]) / trials)
    assert np.all(np.abs(first - P[0]) < 4.5 * sd + 1e-4)
    # given that child c was accepted, the next emitted token follows the target after c
    for c, cnt in second.items():
        m = cnt.sum()
        assert m > 1000
        sdc = np.sqrt(P[c] * (1 - P[c]) / m)
        assert np.all(np.abs(cnt / m - P[c]) < 4.5 * sdc + 1e-4)


def _no_renormalisation(parent, tok, P, u_node, u_bonus):
    n, cur, path = len(parent), 0, [0]
    while True:
        p = np.array(P[cur], dtype=np.float64)
        nxt = None
        for c in range(cur + 1, n):
            if parent[c] != cur:
                continue
            if u_node[c] < p[tok[c]]:
                nxt = c
                break
            p[tok[c]] = 0.0  # mass removed but the rest is not divided by (1 - p(c))
        if nxt is None:
            cdf = np.cumsum(p)
            return np.asarray(path), int(min(np.searchsorted(cdf, u_bonus * cdf[-1], side="right"), len(p) - 1))
        cur = nxt
        path.append(cur)


def _residual_keeps_rejected(parent, tok, P, u_node, u_bonus):
    n, cur, path = len(parent), 0, [0]
    while True:
        p = np.array(P[cur], dtype=np.float64)
        removed = 0.0
        nxt = None
        for c in range(cur + 1, n):
            if parent[c] != cur:
                continue
            if u_node[c] < p[tok[c]] / (1.0 - removed):
                nxt = c
                break
            removed += p[tok[c]]
        if nxt is None:
            cdf = np.cumsum(p)  # the final draw forgets what was rejected
            return np.asarray(path), int(min(np.searchsorted(cdf, u_bonus * cdf[-1], side="right"), len(p) - 1))
        cur = nxt
        path.append(cur)


@pytest.mark.parametrize("wrong", [_no_renormalisation, _residual_keeps_rejected])
def test_planted_mistakes_break_the_distribution(wrong):
    P = _target(1, len(TREE_PARENT), 6)
    trials = 20000
    first, _ = _simulate(wrong, TREE_PARENT, TREE_TOK, P, trials, 7)
    sd = np.sqrt(P[0] * (1 - P[0]) / trials)
    assert np.any(np.abs(first - P[0]) > 6 * sd)


def test_softmax_temperature_limits():
    g = synth.philox(3, 43)
    z = g.standard_normal((4, 50))
    assert np.allclose(orc.softmax_temperature(z, 1.0).sum(axis=1), 1.0)
    import torch
    assert np.allclose(orc.softmax_temperature(z, 0.7), torch.softmax(torch.from_numpy(z) / 0.7, dim=-1).numpy())
    cold = orc.softmax_temperature(z, 1e-4)
    assert np.array_equal(cold.argmax(axis=1), z.argmax(axis=1)) and np.all(cold.max(axis=1) > 1 - 1e-9)
