"""Oracle: the ranking-list baselines of Sec. 3.1-3.2 and the pruning baseline (test infrastructure).

promote(subset; all) (Eq. 5) moves an ordered subset to the front and keeps the
rest in their order.  Max-Rank (Eq. 6-7) promotes the cached experts found among
the first M ranks, then the router's own top-J in front of those.
Cumsum-Threshold (Eq. 8) picks M per token as the shortest prefix of the ranking
whose softmax weights sum to at least p, then applies Max-Rank.  Pruning
(Sec. 4.2) discards the experts ranked h or worse.

Parity unpinned: prune().  The paper prints no worked value for it, and its
rank base is a reading (see prune): the tests pin only what follows from the
definition itself (prefix of the ranking, h = K + 1 is the original routing).
"""
from __future__ import annotations

import numpy as np


def promote(subset, ranking):
    """Eq. 5: subset (already in ranking order) followed by the remaining entries in order."""
    sub = list(subset)
    members = set(sub)
    return sub + [e for e in ranking if e not in members]


def max_rank(ranking, cache, max_rank_m: int, top_j: int):
    """Eq. 7: promote(r[:J]; promote(r[:M] ∩ C; r))."""
    r = list(ranking)
    cached_head = [e for e in r[:max_rank_m] if e in cache]
    r1 = promote(cached_head, r)
    return promote(r[:top_j], r1)


def cumsum_rank(weights_sorted, p: float) -> int:
    """Eq. 8: the smallest M with sum of the M largest weights >= p (at least 1, at most N)."""
    total = 0.0
    for m, w in enumerate(weights_sorted, start=1):
        total += float(w)
        if total >= p:
            return m
    return len(weights_sorted)


def cumsum_threshold(ranking, weights, cache, p: float, top_j: int):
    """Sec. 3.2: Max-Rank with the per-token M of Eq. 8."""
    r = list(ranking)
    m = cumsum_rank([weights[e] for e in r], p)
    return max_rank(r, cache, m, top_j)


def prune(ranking, top_k: int, h: int):
    """Sec. 4.2 pruning baseline: of the top-K, the experts ranked >= h are discarded, ranks counted from 1.

    The paper restricts h to 1 < h <= K.  With ranks counted from 1 that range is exactly the useful one: h = 1
    would discard every expert (hence 1 < h) and h = K still discards the last one, so h - 1 experts are kept.
    (Counted from 0 the bound 1 < h would needlessly exclude "keep one expert", and h = K would prune nothing.)
    h = K + 1 keeps all K: the original routing.  The miss rate stays normalised by K: see pruned_miss_rate.
    """
    assert h >= 2, "h = 1 would discard every expert"
    return list(ranking)[: min(top_k, h - 1)]


def pruned_miss_rate(misses: int, tokens: int, top_k: int) -> float:
    """Sec. 4.2: the pruning baseline's miss rate is normalised by the original K, not by the experts kept."""
    return misses / max(tokens * top_k, 1)
