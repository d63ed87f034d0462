"""Oracle: eviction-policy references on recorded selection traces (test infrastructure).

A trace is a list of tokens, each a list of the K distinct expert ids the token
selected, given in the order the cache is to touch them (Sec. 4.2: descending
router weight, so the highest weight is the first to go among one token's
experts).  Misses are counted per token against the cache before the token
(Eq. 4).  Three independent counters:

  * lru_list_misses   - a recency list kept literally (front = least recent);
  * belady_misses     - evict the resident expert needed farthest in the
                        future (the optimal-eviction reference of Sec. 4.8);
  * min_misses_search - exhaustive search over every eviction choice, for
                        tiny traces, to check Belady's count is the minimum.

The paper sweeps the cache size down to one expert; with capacity < K a token
cannot hold all its experts, so only the most recently touched `capacity`
experts of the token stay (counting mode, used by the cache-size sweep).
"""
from __future__ import annotations

from functools import lru_cache


def lru_list_misses(trace, capacity: int, initial=()):
    """Total misses and the final recency list (least recent first)."""
    order = list(initial)  # least recent ... most recent
    misses = 0
    for token in trace:
        token = list(token)
        misses += sum(1 for e in token if e not in order)
        order = [e for e in order if e not in token]  # selected experts leave their old place
        order.extend(token)  # and become the most recent, in touch order
        if len(order) > capacity:
            order = order[len(order) - capacity :]  # drop from the least-recent end
    return misses, order


def lru_list_lifetimes(trace, capacity: int, initial=()):
    """Stays in memory under the recency-list LRU: (sum, count) of the lengths in tokens of the stays that ended
    by eviction, and the still-open stays as {expert: token it was loaded at} (Sec. 4.6, Table 2 'lifetime')."""
    order = list(initial)
    born = {e: 0 for e in order}
    total = count = 0
    for t, token in enumerate(trace):
        token = list(token)
        for e in token:
            if e not in born:
                born[e] = t
        order = [e for e in order if e not in token] + token
        while len(order) > capacity:
            old = order.pop(0)
            total += t - born.pop(old)
            count += 1
    return total, count, born


def belady_misses(trace, capacity: int, initial=()):
    """Misses under farthest-next-use eviction (never-again first; ties -> lowest id)."""
    trace = [list(tok) for tok in trace]
    k = max((len(t) for t in trace), default=0)
    assert capacity >= k, "optimal eviction is defined here for capacity >= K"
    # next_use[t][e]: first token index > t that selects e (or infinity)
    inf = len(trace) + 1
    cache = set(initial)
    misses = 0
    for t, token in enumerate(trace):
        need = [e for e in token if e not in cache]
        misses += len(need)
        for e in need:
            if len(cache) >= capacity:

                def next_use(c):
                    for u in range(t + 1, len(trace)):
                        if c in trace[u]:
                            return u
                    return inf

                cands = sorted(c for c in cache if c not in token)
                victim = max(cands, key=lambda c: (next_use(c), -c))
                cache.remove(victim)
            cache.add(e)
    return misses


def min_misses_search(trace, capacity: int, initial=()):
    """Minimum total misses over all eviction choices (exponential; tiny traces only)."""
    trace = [tuple(tok) for tok in trace]

    @lru_cache(maxsize=None)
    def best(t, cache):
        if t == len(trace):
            return 0
        token = trace[t]
        cache_set = set(cache)
        need = [e for e in token if e not in cache_set]
        if not need:
            return best(t + 1, cache)

        def place(i, cur):
            if i == len(need):
                return best(t + 1, tuple(sorted(cur)))
            e = need[i]
            if len(cur) < capacity:
                return place(i + 1, cur | {e})
            out = None
            for v in cur:
                if v in token:
                    continue
                r = place(i + 1, (cur - {v}) | {e})
                out = r if out is None else min(out, r)
            return out

        return len(need) + place(0, frozenset(cache_set))

    return best(0, tuple(sorted(initial)))


def sequential_lru_misses(trace, capacity: int):
    """Textbook one-request-at-a-time LRU on the flattened trace (differs from Eq. 4 when a
    not-yet-touched expert of the same token is evicted; equal when K == 1)."""
    from collections import OrderedDict

    cache: OrderedDict = OrderedDict()
    misses = 0
    for token in trace:
        for e in token:
            if e in cache:
                cache.move_to_end(e)
            else:
                misses += 1
                if len(cache) >= capacity:
                    cache.popitem(last=False)
                cache[e] = True
    return misses
