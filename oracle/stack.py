"""Oracle: the glue of the synthetic multi-layer workload (test infrastructure).

Not part of the paper's method: it only defines how the hidden state of the
synthetic stacks moves from layer to layer (a residual add plus an AR(1)
perturbation, then a scale-free RMS normalisation that keeps the router's logit
range alike in every layer).  fp64.
"""
from __future__ import annotations

import numpy as np

RMS_EPS = 1e-6
PERTURB = 0.5


def rmsnorm(h: np.ndarray) -> np.ndarray:
    h = np.asarray(h, np.float64)
    return h / np.sqrt(np.mean(h * h) + RMS_EPS)


def next_hidden(h, y, a_next) -> np.ndarray:
    """h_{l+1} = h_l + y_l + 0.5 * a_{l+1,t}."""
    return np.asarray(h, np.float64) + np.asarray(y, np.float64) + PERTURB * np.asarray(a_next, np.float64)
