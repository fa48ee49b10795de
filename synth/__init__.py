"""Seeded synthetic input generators shared by the tests, the bench and the smoke check.

This package produces inputs only (trees, hidden states, weights, KV caches, draft
probabilities, cost vectors, storage-dtype rounding). It contains none of the method's
arithmetic and imports neither the CPU oracle nor the HIP library.
"""
from .inputs import *  # noqa: F401,F403
from .drafter import draft_iteration  # noqa: F401
