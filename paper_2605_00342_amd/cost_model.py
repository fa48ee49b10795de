"""Cost surface over (verification length, expert union) and its collapse to the table C(k).

Prefix selection divides the expected accepted length by a profiled cost C(k) that depends on
the verification length only (Sec. 3.2.3: an average for that length, not a prediction for the
expert set a particular step activates). What makes the cost of a sparse MoE step grow is the
union of activated experts (Sec. 2.2, Eq. 5), whose size for t tokens App. A gives in closed
form under uniform routing. This module is the host logic between the two: it takes profiling
points (k, mean |union|, milliseconds) measured by evict_profile_cost_union on inputs of
different routing spread, fits the surface  C(k, U) = a + b k + c U  by least squares, and
collapses it to a table over k with the union expected at each k -- measured on the profiling
inputs, or the closed form when no measurement covers that k. The arithmetic (closed form, fit,
collapse, table file) is the library's, behind its evict_cost_*_host entry points; this module only
shapes arrays for them and drives the profiling runs. Nothing here runs per decoding step.
"""
from __future__ import annotations

from typing import Iterable, Optional, Sequence, Tuple

import numpy as np

from . import binding as ev


def _invalid_as_value_error(fn, *args):
    try:
        return fn(*args)
    except ev.EvictError as e:
        raise ValueError(str(e)) from None


def expected_union(t, n_experts: int, top_k: int):
    """Unique experts activated by t tokens under independent uniform routing (App. A)."""
    t = np.asarray(t, np.float64)
    out = np.asarray(_invalid_as_value_error(ev.evict_cost_expected_union_host, n_experts, top_k, t.ravel()), np.float64)
    return out.reshape(t.shape) if t.ndim else float(out[0])


def fit_cost_surface(k: Sequence[float], union: Sequence[float], ms: Sequence[float]) -> Tuple[np.ndarray, float]:
    """Least-squares (a, b, c) of ms ~ a + b k + c U, and the root-mean-square residual.
    Needs at least three points that do not lie on one line in the (k, U) plane."""
    k, union, ms = (np.asarray(v, np.float64).ravel() for v in (k, union, ms))
    coef, rms = _invalid_as_value_error(ev.evict_cost_fit_surface_host, k, union, ms)
    return np.asarray(coef, np.float64), rms


def collapse_cost(coef: np.ndarray, k_max: int, n_experts: int, top_k: int,
                  union_of_k: Optional[Sequence[float]] = None) -> np.ndarray:
    """C(k) = a + b k + c U(k) as float32[k_max + 1], the table evict_select_prefix consumes
    (entry 0 repeats entry 1: no prefix is empty). union_of_k[k] is the union expected at
    length k (entries <= 0 or missing fall back to the closed form of App. A)."""
    return np.asarray(_invalid_as_value_error(ev.evict_cost_collapse_host, np.asarray(coef, np.float64), k_max, n_experts, top_k,
                                              None if union_of_k is None else np.asarray(union_of_k, np.float64)), np.float32)


def table_key(device: str, model: str, dtype: str, n_layers: int, ctx_len: int) -> str:
    """The key a cost table is filed under: a table profiled on another device, model shape, storage type,
    depth or context length does not describe this one's costs."""
    return f"{device}:{model}:{dtype}:L{n_layers}:ctx{ctx_len}".replace(" ", "_")


def save_cost_table(path: str, cost: Sequence[float], key: str) -> None:
    """Writes C(k), k = 0..len(cost)-1, in the library's text format under `key`."""
    _invalid_as_value_error(ev.evict_cost_table_save_host, path, cost, key)


def load_cost_table(path: str, expect_key: Optional[str] = None) -> np.ndarray:
    """Reads a table; with expect_key, a table filed under another key is refused."""
    return np.asarray(_invalid_as_value_error(ev.evict_cost_table_load_host, path, expect_key), np.float32)


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
