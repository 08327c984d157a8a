"""Seeded leaf-weight inputs (no circuit arithmetic lives here)."""
from __future__ import annotations

import numpy as np

P_FLOOR = 1e-6   # draws are clamped to [P_FLOOR, 1-P_FLOOR]: Beta(0.5,0.5) otherwise rounds 1-p to 0 in fp32


def leaf_probs(seed: int, batch: int, num_vars: int, dist=("uniform", 0.0, 1.0)) -> np.ndarray:
    """p[B,V] in fp64.  dist: ("uniform", lo, hi) or ("beta", a, b)."""
    rng = np.random.default_rng(seed)
    if dist[0] == "uniform":
        p = rng.uniform(dist[1], dist[2], size=(batch, num_vars))
    elif dist[0] == "beta":
        p = rng.beta(dist[1], dist[2], size=(batch, num_vars))
    else:
        raise ValueError(dist)
    return np.clip(p, P_FLOOR, 1.0 - P_FLOOR)


def as_inputs(p: np.ndarray, log_domain: bool) -> np.ndarray:
    """The fp32 array handed to the evaluators: p itself, or log p taken in fp64 and rounded once.
    The oracle widens this same fp32 array, so input rounding is charged to neither side."""
    x = np.log(p) if log_domain else p
    return np.ascontiguousarray(x, dtype=np.float32)
