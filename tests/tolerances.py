"""Tolerances of the hidden-state comparisons, in one place.

Single layer: 1e-4 (fp32 storage) / 2e-2 (bf16 storage) relative L2, the bar the benchmark spec sets.
Several layers, both sides running on their own: each layer adds an error of at most the single-layer tolerance
relative to the hidden state (whose norm does not shrink along the residual stream), independent from layer to
layer, so the errors add in quadrature: tolerance x sqrt(depth). Measured on the full-size stacks: 0.055 after 48
Qwen3-shaped layers (bound 0.139), 0.055 after 27 DeepSeek-shaped layers (0.104), 0.10 after 48 layers on 4 x 64
truncated trees (0.139); the growth is close to linear in the depth because it is dominated by near-tie routing
flips (a flipped token keeps diverging), not by rounding.
"""
import math

TOL = {"f32": 1e-4, "bf16": 2e-2}
ROW_FACTOR = 3.0   # worst single token row: at most ROW_FACTOR x the tensor's tolerance (single layer, same routing)


def stack_tol(dtype: str, depth: int) -> float:
    return TOL[dtype] * math.sqrt(max(depth, 1))
