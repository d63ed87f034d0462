"""Pins of the prompt-phase oracle (no GPU): a batch is its tokens in order, and in a stack without cross-token
coupling the layer-by-layer order of the prompt phase gives, per layer, the cache history of the decode order."""
import numpy as np

from oracle import prompt, routing


def _stack(seed, L=3, d=16, N=8, I=12, T=20):
    r = np.random.default_rng(seed)
    gates = [r.normal(size=(N, d)) * 0.5 for _ in range(L)]
    W = {(l, e): dict(gate=r.normal(size=(I, d)) * 0.3, up=r.normal(size=(I, d)) * 0.3, down=r.normal(size=(d, I)) * 0.3)
         for l in range(L) for e in range(N + 1)}
    a = r.normal(size=(T, L, d))
    return gates, W, a


def test_batch_routing_is_token_by_token():
    """B routing steps: identical to stepping the router by hand, including the state it is left in, and it does not
    matter how the prompt is cut into batches."""
    r = np.random.default_rng(5)
    N, K, C, T = 12, 3, 5, 64
    Z = (np.cumsum(r.normal(size=(T, N)), axis=0) * 0.2 + r.normal(size=(T, N))).astype(np.float32)
    whole = routing.CachePriorRouter(N, K, C, 0.5, 1)
    res = prompt.route_batch(whole, Z)
    by_hand = routing.CachePriorRouter(N, K, C, 0.5, 1)
    for t in range(T):
        ref = by_hand.step(Z[t])
        assert res[t].sel.tolist() == ref.sel.tolist() and res[t].miss == ref.miss and res[t].slot == ref.slot
    cut = routing.CachePriorRouter(N, K, C, 0.5, 1)
    pieces = prompt.route_batch(cut, Z[:7]) + prompt.route_batch(cut, Z[7:40]) + prompt.route_batch(cut, Z[40:])
    assert [p.sel.tolist() for p in pieces] == [p.sel.tolist() for p in res]
    assert cut.stats.misses == whole.stats.misses == by_hand.stats.misses
    assert cut.cache.slot_of == whole.cache.slot_of and cut.cache.stamp == whole.cache.stamp


def test_layer_major_prompt_equals_token_major_decode():
    """Every layer sees the same tokens in the same order either way, so selections, miss counts and the final
    outputs agree exactly (same fp64 operations on the same values)."""
    for seed in (1, 2):
        gates, W, a = _stack(seed)
        L, N = len(gates), gates[0].shape[0]
        mk = lambda: [routing.CachePriorRouter(N, 2, 4, 0.5) for _ in range(L)]
        ra, rb = mk(), mk()
        ef, sf = (lambda l, e: W[(l, e)]), (lambda l: W[(l, N)])
        sel_a, Ya = prompt.stack_layer_major(ra, gates, a, ef, sf)
        sel_b, Yb = prompt.stack_token_major(rb, gates, a, ef, sf)
        assert sel_a == sel_b
        np.testing.assert_array_equal(Ya, Yb)
        for x, y in zip(ra, rb):
            assert (x.stats.misses, x.stats.evictions, x.stats.lifetime_sum) == (y.stats.misses, y.stats.evictions,
                                                                                 y.stats.lifetime_sum)
        assert sum(x.stats.misses for x in ra) > 2 * L  # the caches are small enough to be exercised


def test_layer_batch_output_is_eq1_per_token():
    from oracle import experts as oexp

    gates, W, a = _stack(3, L=1)
    N = gates[0].shape[0]
    router = routing.CachePriorRouter(N, 2, 4, 0.0)
    X = a[:, 0].astype(np.float32)
    res, Y = prompt.layer_batch(router, gates[0], X, lambda e: W[(0, e)], W[(0, N)])
    for t in (0, 7, 19):
        z = routing.router_logits(gates[0], X[t])
        top2 = np.argsort(-z, kind="stable")[:2]
        assert res[t].sel.tolist() == top2.tolist()  # lambda = 0: the original routing
        w = routing.softmax(z)[top2]
        y = sum(w[i] * oexp.swiglu_expert(X[t], **W[(0, int(top2[i]))]) for i in range(2)) + oexp.swiglu_expert(X[t], **W[(0, N)])
        np.testing.assert_allclose(Y[t], y, rtol=1e-12)
