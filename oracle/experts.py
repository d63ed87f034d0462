"""Oracle: expert networks and the MoE layer output (test infrastructure).

y = sum_{i in r[:K]} w_i E_i(x) (Eq. 1).  The paper leaves E_i unspecified; the
workloads fix it as a bias-free SwiGLU, E(x) = W_down (silu(W_gate x) * (W_up x)),
and shared experts (Table 1) as one more SwiGLU that is always applied with
weight 1.  All arithmetic is fp64 on the stored weight values; quantised
weights are dequantised from the stored integers and fp16 scales first, so
quantisation error is outside the comparison.
"""
from __future__ import annotations

import numpy as np

f64 = np.float64
INT4_GROUP = 128


def dequantize(w) -> np.ndarray:
    """Stored weight -> fp64 matrix.

    w is a float array, or (q int8 [R,C], s fp16 [R]) per-row int8, or
    (packed uint8 [R,C/2], s fp16 [R,C/128]) group-128 int4 with nibble = q + 8 and the
    even column in the low nibble.
    """
    if not isinstance(w, tuple):
        return np.asarray(w, f64)
    q, s = w
    q = np.asarray(q)
    s = np.asarray(s, f64)
    if q.dtype == np.int8:
        return q.astype(f64) * s[:, None]
    assert q.dtype == np.uint8
    rows, half = q.shape
    full = np.empty((rows, 2 * half), f64)
    full[:, 0::2] = (q & 15).astype(f64) - 8.0
    full[:, 1::2] = (q >> 4).astype(f64) - 8.0
    return full * np.repeat(s, INT4_GROUP, axis=1)


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def swiglu_expert(x, gate, up, down) -> np.ndarray:
    """E(x) = W_down (silu(W_gate x) * (W_up x)); gate/up are [I,d], down is [d,I]."""
    x = np.asarray(x, f64)
    h = silu(dequantize(gate) @ x) * (dequantize(up) @ x)
    return dequantize(down) @ h


def moe_output(x, experts, weights, shared=None) -> np.ndarray:
    """Eq. 1 over the selected experts (dicts with 'gate','up','down'), plus the shared expert."""
    x = np.asarray(x, f64)
    y = np.zeros(x.shape[0], f64)
    for w, e in zip(weights, experts):
        y += float(w) * swiglu_expert(x, e["gate"], e["up"], e["down"])
    if shared is not None:
        y += swiglu_expert(x, shared["gate"], shared["up"], shared["down"])
    return y


def rel_err(got, ref) -> float:
    """max_j |got - ref| / max_j |ref| (element-wise ratios blow up near zero)."""
    got = np.asarray(got, f64)
    ref = np.asarray(ref, f64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))
