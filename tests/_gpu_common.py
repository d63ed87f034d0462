"""Helpers for the GPU parity tests: build a store from synthetic weights, hand the same values to the oracle."""
from __future__ import annotations

import numpy as np
import torch

from synth import workloads

DEV = "cuda:0"


def to_np(w):
    """Stored weight (tensor or (q, scale)) -> numpy values for the oracle (bf16 widened exactly to fp32)."""
    if isinstance(w, tuple):
        return tuple(to_np(t) for t in w)
    if w.dtype == torch.bfloat16:
        w = w.float()
    return w.detach().cpu().numpy()


def np_expert(weights: dict) -> dict:
    return {k: to_np(v) for k, v in weights.items()}


def build(cfg, *, lam=0.0, top_j=None, initial=None, delta_fixed=None, delta_per_token=False, route_mode=0,
          max_rank=0, cumsum_p=0.0):
    import paper_2412_00099_amd as pkg

    store = pkg.ExpertStore(
        n_layers=cfg.n_layers, hidden=cfg.hidden, n_experts=cfg.n_experts, inter=cfg.inter,
        shared_inter=cfg.shared_inter, capacity=cfg.capacity, weight_fmt=cfg.weight_fmt, act_fmt=cfg.act_fmt,
        device=DEV,
    )
    store.fill_from(cfg, workloads.expert_weights, workloads.shared_weights, workloads.gate_weight)
    dec = pkg.MoEDecoder(
        store, top_k=cfg.top_k, top_j=cfg.top_j if top_j is None else top_j, lam=lam,
        renormalize=cfg.renormalize, initial=initial, delta_fixed=delta_fixed, delta_per_token=delta_per_token,
        route_mode=route_mode, max_rank=max_rank, cumsum_p=cumsum_p,
    )
    return store, dec


class OracleWeights:
    """Canonical weights regenerated on the CPU from the same seeds (cached per (layer, expert))."""

    def __init__(self, cfg):
        self.cfg = cfg
        self._cache = {}

    def expert(self, layer, e):
        key = (layer, e)
        if key not in self._cache:
            if len(self._cache) > 64:
                self._cache.clear()
            self._cache[key] = np_expert(workloads.expert_weights(self.cfg, layer, e, "cpu"))
        return self._cache[key]

    def shared(self, layer):
        if not self.cfg.shared_inter:
            return None
        key = (layer, "shared")
        if key not in self._cache:
            self._cache[key] = np_expert(workloads.shared_weights(self.cfg, layer, "cpu"))
        return self._cache[key]

    def gate(self, layer):
        key = (layer, "gate")
        if key not in self._cache:
            self._cache[key] = to_np(workloads.gate_weight(self.cfg, layer, "cpu"))
        return self._cache[key]


def route_fields(out, k):
    return dict(
        sel=list(out.sel_expert[:k]), slot=list(out.sel_slot[:k]), miss=[bool(m) for m in out.miss[:k]],
        evicted=list(out.evicted[:k]), weight=np.array(out.sel_weight[:k], np.float64), n_miss=out.n_miss,
        token=out.token, delta=np.float32(out.delta), margin=out.margin,
    )


def check_tables(dec, layer, router, n_experts, capacity):
    """Slot table, stamps, Delta accumulator and counters of one layer against the oracle router: exact."""
    t = dec.tables(layer)
    cache = router.cache
    assert list(t.expert_slot[:n_experts]) == cache.slot_of
    assert list(t.slot_expert[:capacity]) == cache.expert_in
    for e in range(n_experts):
        if cache.slot_of[e] >= 0:
            assert t.stamp[e] == cache.stamp[e], (e, t.stamp[e], cache.stamp[e])
    assert np.float32(t.delta_sum) == router.range.total
    assert t.count == router.range.count
    s = dec.stats(layer)
    o = router.stats
    assert (s.tokens, s.selections, s.hits, s.misses, s.cold_misses, s.evictions, s.lifetime_sum) == (
        o.tokens, o.selections, o.hits, o.misses, o.cold_misses, o.evictions, o.lifetime_sum)
