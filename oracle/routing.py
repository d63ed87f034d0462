"""Oracle: router, Cache-Prior re-ranking and the LRU expert cache (test infrastructure).

Follows Sec. 2.1 (Eq. 1-3: logits z = G(x), weights w = softmax(z), ranking
r = argsort w, top-K), Sec. 2.2 (Eq. 4: hit rate against the cache at selection
time), Sec. 3.3 (Eq. 9: z' = z + lambda * Delta_avg * m~_t; Eq. 10: Delta_avg, the
running mean of max(z) - min(z); the optional top-J guarantee) and Sec. 4.2
(LRU eviction, with the experts of one token ordered so that higher router
weights are evicted first).

Cache-Prior is a heuristic whose result is defined by its steps, so the steps
are taken here in the paper's order.  Steps that decide an integer (which
expert, which slot) are carried out in fp32 with one rounding per operation,
the precision the router logits are produced in; everything else is fp64.

Readings where the paper is silent (also listed in the design notes):
  * ties in any ranking go to the lower expert index;
  * Delta_avg is the cumulative arithmetic mean including the current token;
  * misses are counted per token against the cache as it stood before the
    token (Eq. 4); experts selected by the token are never evicted by it;
  * recency stamp of the expert at position p (by descending original logit)
    of token t is t*K + p, so within a token the highest weight is the oldest.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

f32 = np.float32
f64 = np.float64


def router_logits(gate_w: np.ndarray, x: np.ndarray) -> np.ndarray:
    """z = G(x) = W_gate x (Eq. 3), accumulated in fp64, returned as fp32."""
    return (np.asarray(gate_w, f64) @ np.asarray(x, f64)).astype(f32)


def softmax(z: np.ndarray) -> np.ndarray:
    """w = sigma(z) (Eq. 3) in fp64."""
    z = np.asarray(z, f64)
    e = np.exp(z - z.max())
    return e / e.sum()


def ranking(v: np.ndarray) -> np.ndarray:
    """r = argsort(v) in descending order (Eq. 2); equal values keep index order."""
    return np.argsort(-np.asarray(v), kind="stable")


class LogitRange:
    """Delta_avg of Eq. 10 as a running mean over tokens (fp32, one rounding per step).  Two variants of the
    estimate (App. D discusses the choice): a fixed value, e.g. from a calibration set, and the current token's
    own range max z - min z with no averaging at all."""

    def __init__(self, fixed: float | None = None, per_token: bool = False):
        assert fixed is None or not per_token
        self.fixed = None if fixed is None else f32(fixed)
        self.per_token = per_token
        self.total = f32(0.0)
        self.count = 0

    def update(self, z: np.ndarray) -> np.float32:
        z = np.asarray(z, f32)
        rng = f32(z.max() - z.min())
        self.total = f32(self.total + rng)
        self.count += 1
        if self.fixed is not None:
            return self.fixed
        if self.per_token:
            return rng
        return f32(self.total / f32(self.count))


def cache_prior_logits(z, mask, lam, delta) -> np.ndarray:
    """z' = z + lambda * Delta_avg * m~ (Eq. 9) in fp32: bias rounded once, one add per expert."""
    z = np.asarray(z, f32)
    bias = f32(f32(lam) * f32(delta))
    return np.where(np.asarray(mask, bool), (z + bias).astype(f32), z)


def guaranteed_mask(z, resident_mask, top_j: int) -> np.ndarray:
    """m~_t: the cache bitmask with the router's own top-J experts OR-ed in (Sec. 3.3)."""
    m = np.array(resident_mask, bool, copy=True)
    if top_j > 0:
        m[ranking(z)[:top_j]] = True
    return m


def cache_prior_select(z, resident_mask, lam, delta, top_k: int, top_j: int = 0) -> np.ndarray:
    """Expert ids r'[:K], ranked by the manipulated logits z' (Sec. 3.3)."""
    zp = cache_prior_logits(z, guaranteed_mask(z, resident_mask, top_j), lam, delta)
    return ranking(zp)[:top_k]


def expert_weights(z, sel, renormalize: bool) -> np.ndarray:
    """w[sel] from the UNMODIFIED logits (Sec. 3.3), optionally renormalised over the K (Sec. 2.1)."""
    w = softmax(z)[np.asarray(sel)]
    return w / w.sum() if renormalize else w


@dataclass
class CacheStats:
    tokens: int = 0
    selections: int = 0
    hits: int = 0
    misses: int = 0
    cold_misses: int = 0
    evictions: int = 0
    lifetime_sum: int = 0  # over evicted experts: tokens between being loaded and being evicted

    @property
    def miss_rate(self) -> float:
        return self.misses / max(self.selections, 1)

    @property
    def mean_lifetime(self) -> float:
        """Average number of time steps an expert stays in memory (Sec. 4.6, Table 2), over completed stays."""
        return self.lifetime_sum / max(self.evictions, 1)


class ExpertCache:
    """C expert slots with LRU eviction by recency stamps (Sec. 4.2)."""

    def __init__(self, n_experts: int, capacity: int, initial=()):
        self.n, self.c = n_experts, capacity
        self.slot_of = [-1] * n_experts  # expert -> slot
        self.expert_in = [-1] * capacity  # slot -> expert
        self.stamp = [0] * n_experts  # valid while resident
        self.ever_used = [False] * capacity
        self.born = [0] * n_experts  # token index at which the expert was loaded (initial residents: 0)
        self.stats = CacheStats()
        initial = list(initial)
        assert len(initial) <= capacity and len(set(initial)) == len(initial)
        for i, e in enumerate(initial):
            self.slot_of[e] = i
            self.expert_in[i] = e
            self.stamp[e] = i - len(initial)  # -n .. -1 in list order
            self.ever_used[i] = True

    def resident_mask(self) -> np.ndarray:
        return np.array([s >= 0 for s in self.slot_of], bool)

    def residents(self) -> set:
        return {e for e in range(self.n) if self.slot_of[e] >= 0}

    def access(self, sel, z):
        """Account one token's selection (Eq. 4) and update the cache.

        sel: selected expert ids in ranked order; z: original logits.
        Returns (miss flag per entry of sel, slot per entry of sel, evicted expert per
        entry of sel or -1).
        """
        sel = [int(e) for e in sel]
        k = len(sel)
        assert k <= self.c and len(set(sel)) == k
        t = self.stats.tokens
        miss = [self.slot_of[e] < 0 for e in sel]
        # order of the token's experts: descending original logit, ties -> lower index
        z = np.asarray(z, f32)
        order = sorted(sel, key=lambda e: (-float(z[e]), e))
        for p, e in enumerate(order):
            self.stamp[e] = t * k + p
        evicted = {}
        for e in order:
            if self.slot_of[e] >= 0:
                continue
            empty = [s for s in range(self.c) if self.expert_in[s] < 0]
            if empty:
                s = empty[0]
                if not self.ever_used[s]:
                    self.stats.cold_misses += 1
                evicted[e] = -1
            else:
                s = min(range(self.c), key=lambda q: self.stamp[self.expert_in[q]])
                old = self.expert_in[s]
                assert old not in sel, "a selected expert may never be a victim"
                self.slot_of[old] = -1
                evicted[e] = old
                self.stats.evictions += 1
                self.stats.lifetime_sum += t - self.born[old]
            self.born[e] = t
            self.expert_in[s] = e
            self.slot_of[e] = s
            self.ever_used[s] = True
        self.stats.tokens += 1
        self.stats.selections += k
        self.stats.misses += sum(miss)
        self.stats.hits += k - sum(miss)
        return miss, [self.slot_of[e] for e in sel], [evicted.get(e, -1) for e in sel]


@dataclass
class RouteResult:
    sel: np.ndarray  # [K] expert ids, ranked by z'
    weight: np.ndarray  # [K] fp64 weights from unmodified z
    miss: list
    slot: list
    evicted: list
    delta: np.float32
    z_prime: np.ndarray = field(repr=False, default=None)


class CachePriorRouter:
    """One MoE layer's router state: Delta_avg accumulator + expert cache, stepped token by token."""

    def __init__(self, n_experts, top_k, capacity, lam, top_j=0, renormalize=False, initial=(), delta_fixed=None,
                 delta_per_token=False):
        assert 0 <= top_j <= top_k <= capacity <= n_experts
        self.n, self.k, self.j = n_experts, top_k, top_j
        self.lam = lam
        self.renormalize = renormalize
        self.range = LogitRange(delta_fixed, delta_per_token)
        self.cache = ExpertCache(n_experts, capacity, initial)

    def select(self, z):
        """Steps up to the selection, without touching the cache: returns (sel, z', delta)."""
        z = np.asarray(z, f32)
        assert z.shape == (self.n,) and np.all(np.isfinite(z))
        delta = self.range.update(z)
        mask = guaranteed_mask(z, self.cache.resident_mask(), self.j)
        zp = cache_prior_logits(z, mask, self.lam, delta)
        return ranking(zp)[: self.k], zp, delta

    def commit(self, z, sel, zp=None, delta=None) -> RouteResult:
        w = expert_weights(z, sel, self.renormalize)
        miss, slot, ev = self.cache.access(sel, z)
        return RouteResult(np.asarray(sel), w, miss, slot, ev, delta, zp)

    def step(self, z) -> RouteResult:
        sel, zp, delta = self.select(z)
        return self.commit(z, sel, zp, delta)

    @property
    def stats(self) -> CacheStats:
        return self.cache.stats


def topk_margin(zp: np.ndarray, top_k: int) -> float:
    """Gap between the K-th and (K+1)-th largest manipulated logit (for tie logging)."""
    s = np.sort(np.asarray(zp, f64))[::-1]
    return float(s[top_k - 1] - s[top_k]) if top_k < len(s) else float("inf")
