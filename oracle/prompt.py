"""Oracle: a batch of prompt tokens through one MoE layer, and through a stack (test infrastructure).

The paper applies its routing during generation and leaves prompt processing to batched kernels (Sec. 4.5; App. F
varies the prompt length); it does not say how the cache is consulted inside a batch.  Reading taken here: the cache
bitmask m_t of Sec. 3.3 is by definition the state of the cache after token t-1, so a batch is routed as its tokens
one after the other - the selections, the LRU updates (Sec. 4.2), Delta_avg (Eq. 10) and the misses of Eq. 4 are those
of the same tokens fed one by one.  Batching changes the schedule of the arithmetic, not a single decision, and the
layer output of every token is Eq. 1 on its own selection.

In the synthetic stacks a token's hidden state depends only on that token's own outputs in earlier layers (no
attention), so sending all tokens through layer l before layer l + 1 gives the same cache states per layer - each
layer sees the same tokens in the same order - as sending token after token through the whole stack.
"""
from __future__ import annotations

import numpy as np

from . import experts as oexp
from . import routing, stack


def route_batch(router: routing.CachePriorRouter, logits) -> list:
    """Route the rows of `logits` ([B, N]) in order: B routing steps of Sec. 3.3, one RouteResult per token."""
    return [router.step(z) for z in np.asarray(logits, np.float32)]


def layer_batch(router, gate_w, X, expert_fn, shared=None):
    """Tokens X [B, d] through one layer: logits (Eq. 3), routing in token order, outputs (Eq. 1).

    expert_fn(e) returns the weights of expert e.  Returns (results, Y [B, d] fp64)."""
    X = np.asarray(X)
    results, Y = [], np.zeros(X.shape, np.float64)
    for t in range(X.shape[0]):
        res = router.step(routing.router_logits(gate_w, X[t]))
        Y[t] = oexp.moe_output(X[t], [expert_fn(int(e)) for e in res.sel], res.weight, shared)
        results.append(res)
    return results, Y


def stack_layer_major(routers, gates, a, expert_fn, shared_fn, act_round=lambda v: v):
    """A prompt of T tokens through an L-layer synthetic stack, layer by layer (all tokens through layer l, then
    l + 1).  a: [T, L, d] perturbation streams (see oracle.stack).  expert_fn(l, e), shared_fn(l) give weights;
    act_round rounds activations to the activation type.  Returns selections [L][T] and the last layer's outputs."""
    T, L, d = a.shape
    H = np.asarray(a[:, 0], np.float64).copy()
    sel, Y = [], None
    for l in range(L):
        X = np.stack([act_round(stack.rmsnorm(H[t]).astype(np.float32)) for t in range(T)])
        res, Y = layer_batch(routers[l], gates[l], X, lambda e, l=l: expert_fn(l, e), shared_fn(l))
        sel.append([r.sel.tolist() for r in res])
        if l + 1 < L:
            H = np.stack([stack.next_hidden(H[t], Y[t], a[t, l + 1]) for t in range(T)])
    return sel, Y


def stack_token_major(routers, gates, a, expert_fn, shared_fn, act_round=lambda v: v):
    """The same stack, token after token through all layers (the decode order)."""
    T, L, d = a.shape
    sel = [[None] * T for _ in range(L)]
    Y = np.zeros((T, d), np.float64)
    for t in range(T):
        h = np.asarray(a[t, 0], np.float64)
        for l in range(L):
            x = act_round(stack.rmsnorm(h).astype(np.float32))
            res = routers[l].step(routing.router_logits(gates[l], x))
            y = oexp.moe_output(x, [expert_fn(l, int(e)) for e in res.sel], res.weight, shared_fn(l))
            sel[l][t] = res.sel.tolist()
            if l + 1 < L:
                h = stack.next_hidden(h, y, a[t, l + 1])
        Y[t] = y
    return sel, Y
