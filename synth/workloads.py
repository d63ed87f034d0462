"""Seeded synthetic MoE workloads: shapes, weights, quantised weights, AR(1) inputs.

These stand in for the paper's trained models and text (Table 1 gives the
expert counts, top-k and parameters per expert the shapes follow; the default
cache is half the experts, Sec. 4.3 / App. D).  Weights are i.i.d. normal with
standard deviation 0.02; hidden states follow a stationary AR(1) process so
that consecutive tokens pick overlapping experts.

The module only produces inputs.  Quantisation is input preparation too: the
paper names 4-bit and 8-bit weights (Sec. 4.5) without a format, so the format
is fixed here once and both the oracle and the HIP library receive the same
stored integers and scales.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch

from . import rng

WEIGHT_STD = 0.02
INT4_GROUP = 128


@dataclass(frozen=True)
class MoEWorkload:
    name: str
    n_layers: int
    hidden: int
    n_experts: int
    inter: int
    shared_inter: int
    top_k: int
    capacity: int
    weight_fmt: str  # 'fp32' | 'bf16' | 'int8' | 'int4'
    act_fmt: str  # 'fp32' | 'bf16'
    n_tokens: int
    rho: float
    seed: int
    top_j: int = 0
    renormalize: bool = False

    def with_(self, **kw) -> "MoEWorkload":
        return replace(self, **kw)

    @property
    def act_dtype(self) -> torch.dtype:
        return torch.float32 if self.act_fmt == "fp32" else torch.bfloat16


# The five workload shapes (index = config number - 1).
CONFIGS = {
    "c1_single_fp32": MoEWorkload("c1_single_fp32", 1, 256, 16, 512, 0, 2, 8, "fp32", "fp32", 256, 0.9, 2025),
    "c2_qwen_bf16": MoEWorkload("c2_qwen_bf16", 24, 2048, 60, 1408, 5632, 4, 30, "bf16", "bf16", 1024, 0.9, 2026),
    "c3_olmoe_bf16": MoEWorkload("c3_olmoe_bf16", 16, 2048, 64, 1024, 0, 8, 32, "bf16", "bf16", 2048, 0.8, 2027),
    "c4_dsv2lite_int4": MoEWorkload("c4_dsv2lite_int4", 27, 2048, 64, 1408, 2816, 6, 32, "int4", "bf16", 2048, 0.9, 2028),
    "c5_mixtral_int8": MoEWorkload(
        "c5_mixtral_int8", 32, 4096, 8, 14336, 0, 2, 4, "int8", "bf16", 4096, 0.9, 2029, renormalize=True
    ),
}

# stream ids inside one workload seed
_S_GATE, _S_EXPERT, _S_HIDDEN, _S_LOGITS, _S_MISC = 1, 2, 3, 4, 5


def _normal(cfg: MoEWorkload, ids, n: int, device) -> torch.Tensor:
    return rng.standard_normal(rng.stream_key(cfg.seed, *ids), n, device)


def gate_weight(cfg: MoEWorkload, layer: int, device="cpu") -> torch.Tensor:
    """Router matrix [N, d] in the activation dtype."""
    w = _normal(cfg, (_S_GATE, layer), cfg.n_experts * cfg.hidden, device) * WEIGHT_STD
    return w.view(cfg.n_experts, cfg.hidden).to(cfg.act_dtype)


def _nearest_code(w: torch.Tensor, s: torch.Tensor, lo: int, hi: int) -> torch.Tensor:
    """Integer code q in [lo, hi] minimising |w - q*s| (ties -> smaller q), as an int16 tensor.

    A first guess comes from a division, whose last bit may depend on the device; the decision among the
    guess and its two neighbours is then taken on |w - q*s| evaluated in fp64, where the product and the
    difference are exact, so every device returns the same codes.
    """
    q = torch.clamp(torch.round(w / s), lo, hi)
    w64, s64 = w.double(), s.double()
    err = (w64 - q.double() * s64).abs()
    for dq in (-1.0, 1.0):
        q1 = torch.clamp(q + dq, lo, hi)
        e1 = (w64 - q1.double() * s64).abs()
        better = (e1 < err) | ((e1 == err) & (q1 < q))
        q = torch.where(better, q1, q)
        err = torch.where(better, e1, err)
    return q.to(torch.int16)


def quantize_int8(w: torch.Tensor):
    """Per output row symmetric int8: s = max|w|/127 (stored fp16), q = nearest code in [-127, 127]."""
    s = (w.abs().amax(dim=1) * (1.0 / 127.0)).to(torch.float16)
    s = torch.where(s == 0, torch.ones_like(s), s)
    q = _nearest_code(w, s.float()[:, None], -127, 127).to(torch.int8)
    return q, s


def quantize_int4(w: torch.Tensor):
    """Group-128 symmetric int4 along each row: s = max|w|/7 (fp16), q = nearest code in [-8, 7].

    Stored as one byte per two weights: nibble = q + 8, even column in the low nibble.
    """
    rows, cols = w.shape
    assert cols % INT4_GROUP == 0
    g = w.view(rows, cols // INT4_GROUP, INT4_GROUP)
    s = (g.abs().amax(dim=2) * (1.0 / 7.0)).to(torch.float16)
    s = torch.where(s == 0, torch.ones_like(s), s)
    q = _nearest_code(g, s.float()[:, :, None], -8, 7) + 8
    q = q.view(rows, cols)
    packed = (q[:, 0::2] | (q[:, 1::2] << 4)).to(torch.uint8)
    return packed, s


def _store(cfg: MoEWorkload, w: torch.Tensor):
    if cfg.weight_fmt == "fp32":
        return w
    if cfg.weight_fmt == "bf16":
        return w.to(torch.bfloat16)
    if cfg.weight_fmt == "int8":
        return quantize_int8(w)
    if cfg.weight_fmt == "int4":
        return quantize_int4(w)
    raise ValueError(cfg.weight_fmt)


def expert_weights(cfg: MoEWorkload, layer: int, expert: int, device="cpu", inter: int | None = None):
    """Canonical weights of one SwiGLU expert.

    Returns {'gate': [I,d], 'up': [I,d], 'down': [d,I]} where each entry is a
    tensor (fp32/bf16) or a (q, scale) pair (int8/int4).  expert == n_experts
    addresses the shared expert (pass inter=cfg.shared_inter).
    """
    inter = cfg.inter if inter is None else inter
    d = cfg.hidden
    n = inter * d
    v = _normal(cfg, (_S_EXPERT, layer, expert), 3 * n, device) * WEIGHT_STD
    return {
        "gate": _store(cfg, v[:n].view(inter, d)),
        "up": _store(cfg, v[n : 2 * n].view(inter, d)),
        "down": _store(cfg, v[2 * n :].view(d, inter)),
    }


def shared_weights(cfg: MoEWorkload, layer: int, device="cpu"):
    assert cfg.shared_inter > 0
    return expert_weights(cfg, layer, cfg.n_experts, device, inter=cfg.shared_inter)


def ar1_stream(cfg: MoEWorkload, n_tokens: int | None = None, device="cpu", n_layers: int | None = None):
    """Stationary AR(1) streams a[t, l, :] = rho*a[t-1, l, :] + sqrt(1-rho^2)*eps, a[0] ~ N(0, I).

    fp32, shape [T, L, d].  Each operation is rounded once (no fused multiply-add),
    so the values do not depend on the device.
    """
    T = cfg.n_tokens if n_tokens is None else n_tokens
    L = cfg.n_layers if n_layers is None else n_layers
    d = cfg.hidden
    eps = _normal(cfg, (_S_HIDDEN,), T * L * d, device).view(T, L, d)
    rho = torch.tensor(cfg.rho, dtype=torch.float32, device=device)
    c = torch.tensor(math.sqrt(1.0 - cfg.rho * cfg.rho), dtype=torch.float32, device=device)
    out = torch.empty_like(eps)
    prev = eps[0].clone()
    out[0] = prev
    for t in range(1, T):
        a = prev * rho
        b = eps[t] * c
        prev = a + b
        out[t] = prev
    return out


def logits_stream(cfg: MoEWorkload, n_tokens: int, layer: int = 0, scale: float = 1.0, device="cpu"):
    """AR(1) router logits [T, N] fp32 for tests that feed logits directly."""
    T, N = n_tokens, cfg.n_experts
    eps = _normal(cfg, (_S_LOGITS, layer), T * N, device).view(T, N)
    rho = torch.tensor(cfg.rho, dtype=torch.float32, device=device)
    c = torch.tensor(math.sqrt(1.0 - cfg.rho * cfg.rho), dtype=torch.float32, device=device)
    out = torch.empty_like(eps)
    prev = eps[0].clone()
    out[0] = prev
    for t in range(1, T):
        prev = prev * rho + eps[t] * c  # two roundings: mul then add (no fma in eager torch)
        out[t] = prev
    return out * torch.tensor(scale, dtype=torch.float32, device=device)


def initial_residents(cfg: MoEWorkload, layer: int, count: int):
    """A seeded random set of `count` distinct experts (App. G: random initial cache)."""
    key = rng.stream_key(cfg.seed, _S_MISC, layer)
    scores = rng.random_bits(key, cfg.n_experts)
    return torch.argsort(scores, stable=True)[:count].tolist()
