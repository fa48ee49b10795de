"""Cost surface over (verification length, expert union) and its collapse to the table C(k).

Prefix selection divides the expected accepted length by a profiled cost C(k) that depends on
the verification length only (Sec. 3.2.3: an average for that length, not a prediction for the
expert set a particular step activates). What makes the cost of a sparse MoE step grow is the
union of activated experts (Sec. 2.2, Eq. 5), whose size for t tokens App. A gives in closed
form under uniform routing. This module is the host logic between the two: it takes profiling
points (k, mean |union|, milliseconds) measured by evict_profile_cost_union on inputs of
different routing spread, fits the surface  C(k, U) = a + b k + c U  by least squares, and
collapses it to a table over k with the union expected at each k -- measured on the profiling
inputs, or the closed form when no measurement covers that k. Plain numpy on a few hundred
points; nothing here runs per decoding step.
"""
from __future__ import annotations

from typing import Iterable, Optional, Sequence, Tuple

import numpy as np

from . import binding as ev


def expected_union(t, n_experts: int, top_k: int):
    """Unique experts activated by t tokens under independent uniform routing (App. A):
    M (1 - (1 - K/M)^t)."""
    t = np.asarray(t, np.float64)
    return n_experts * (1.0 - (1.0 - top_k / n_experts) ** t)


def fit_cost_surface(k: Sequence[float], union: Sequence[float], ms: Sequence[float]) -> Tuple[np.ndarray, float]:
    """Least-squares (a, b, c) of ms ~ a + b k + c U, and the root-mean-square residual.
    Needs at least three points that do not lie on one line in the (k, U) plane."""
    k, union, ms = (np.asarray(v, np.float64).ravel() for v in (k, union, ms))
    if not (k.size == union.size == ms.size) or k.size < 3:
        raise ValueError("fit_cost_surface: need >= 3 points with k, union and ms of one length")
    A = np.stack([np.ones_like(k), k, union], axis=1)
    if np.linalg.matrix_rank(A) < 3:
        raise ValueError("fit_cost_surface: the (k, union) points lie on one line; profile inputs of another routing spread")
    coef, *_ = np.linalg.lstsq(A, ms, rcond=None)
    rms = float(np.sqrt(np.mean((A @ coef - ms) ** 2)))
    return coef, rms


def cost_surface(coef: np.ndarray, k_max: int, n_experts: int) -> np.ndarray:
    """The fitted surface as a table float32[k_max + 1][n_experts + 1] over (k, U)."""
    kk, uu = np.meshgrid(np.arange(k_max + 1), np.arange(n_experts + 1), indexing="ij")
    return (coef[0] + coef[1] * kk + coef[2] * uu).astype(np.float32)


def collapse_cost(coef: np.ndarray, k_max: int, n_experts: int, top_k: int,
                  union_of_k: Optional[Sequence[float]] = None) -> np.ndarray:
    """C(k) = a + b k + c U(k) as float32[k_max + 1], the table evict_select_prefix consumes
    (entry 0 repeats entry 1: no prefix is empty). union_of_k[k] is the union expected at
    length k (entries <= 0 or missing fall back to the closed form of App. A)."""
    u = expected_union(np.arange(k_max + 1), n_experts, top_k)
    if union_of_k is not None:
        m = np.asarray(union_of_k, np.float64)
        n = min(m.size, k_max + 1)
        u[:n] = np.where(m[:n] > 0, m[:n], u[:n])
    cost = coef[0] + coef[1] * np.arange(k_max + 1) + coef[2] * u
    cost[0] = cost[1] if k_max >= 1 else cost[0]
    if not np.all(cost > 0):
        raise ValueError("collapse_cost: the fitted surface is not positive over the table's range")
    return cost.astype(np.float32)


def profile_cost_surface(ctx, layers, input_sets: Iterable[dict], k_max: int, reps: int):
    """Runs evict_profile_cost_union once per input set (each a dict with tree_off, parent,
    k_caches, v_caches, kv_head_stride, ctx_len, max_ctx_host, x_in, x_out, k_new, v_new: device
    tensors / lists as the entry point takes them) and returns (k, union, ms) arrays of all points
    plus the mean union per k over the sets (float64[k_max + 1], entry 0 = 0)."""
    ks, us, ts = [], [], []
    mean_u = np.zeros(k_max + 1)
    n_sets = 0
    for s in input_sets:
        cost, umean = ev.evict_profile_cost_union(ctx, layers, s["tree_off"], s["parent"], k_max, s["k_caches"], s["v_caches"],
                                                  s["kv_head_stride"], s["ctx_len"], s["max_ctx_host"], s["x_in"], s["x_out"],
                                                  s["k_new"], s["v_new"], reps)
        ks += list(range(1, k_max + 1))
        us += umean[1:]
        ts += cost[1:]
        mean_u += np.asarray(umean)
        n_sets += 1
    if n_sets == 0:
        raise ValueError("profile_cost_surface: no input set")
    return np.asarray(ks, np.float64), np.asarray(us, np.float64), np.asarray(ts, np.float64), mean_u / n_sets
