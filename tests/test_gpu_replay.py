"""Full-length routing replay: every workload at its full depth, expert count, top-K, cache size and token count,
driven exactly as bench.py drives it (non-blocking layer boundary, expert output left pending, fills on the side
stream), with every routing step's record fetched from the device.  The logits the device used are then replayed
through the oracle router, layer by layer, and everything that is an integer must be identical: ranked expert
ids, slots, miss flags, evicted experts, the final slot tables, stamps and all counters; Delta_avg bit for bit;
weights to fp32 rounding.  Replaying the device's own fp32 logits makes the comparison immune to bf16 drift of
the residual stream, and no oracle input other than those logits comes from the device.

The benchmarked workload runs at its real shape (so the miss counts bench.py prints are these, kernels being
deterministic); the other three keep L, N, K, C, T and the hidden size but use a small expert intermediate size -
the routing state does not depend on it - so that the host tier stays small."""
import numpy as np
import pytest
import torch

from oracle import routing, stack
from synth import workloads
from synth.workloads import CONFIGS

from _gpu_common import DEV, build, check_tables

pytestmark = pytest.mark.gpu


def replay_case(cfg, lam, T, warmup=0):
    L, N, K, C = cfg.n_layers, cfg.n_experts, cfg.top_k, cfg.capacity
    print(f"case replay {cfg.name} L={L} N={N} K={K} C={C} I={cfg.inter} T={T} lam={lam}", flush=True)
    store, dec = build(cfg, lam=lam)
    a = workloads.ar1_stream(cfg, T, device=DEV)
    h = torch.zeros(cfg.hidden, dtype=torch.float32, device=DEV)
    x = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()
    logits = np.zeros((T, L, N), np.float32)
    ints = np.zeros((T, L, 4, K), np.int32)  # expert, slot, miss, evicted
    weight = np.zeros((T, L, K), np.float32)
    delta = np.zeros((T, L), np.float32)
    for t in range(T):
        if t % 256 == 0:
            print(f"  device token {t}", flush=True)
        for l in range(L):
            dec.stack_route_step(l, h, a[t, l], 1.0 if l == 0 else stack.PERTURB, x, carry=l > 0, wait=False)
            dec.expert_forward(l, x, None)
            r = dec.last_route(l)
            assert r.token == t
            logits[t, l] = r.logits[:N]
            ints[t, l, 0], ints[t, l, 1] = r.sel_expert[:K], r.sel_slot[:K]
            ints[t, l, 2], ints[t, l, 3] = r.miss[:K], r.evicted[:K]
            weight[t, l] = r.sel_weight[:K]
            delta[t, l] = r.delta
    dec.compute_stream.synchronize()
    assert np.all(np.isfinite(logits))
    total = steady = 0
    for l in range(L):
        router = routing.CachePriorRouter(N, K, C, lam, cfg.top_j, cfg.renormalize)
        for t in range(T):
            ref = router.step(logits[t, l])
            ctx = f"{cfg.name} lam={lam} token {t} layer {l}"
            assert ints[t, l, 0].tolist() == ref.sel.tolist(), ctx
            assert ints[t, l, 1].tolist() == ref.slot, ctx
            assert [bool(m) for m in ints[t, l, 2]] == ref.miss, ctx
            assert ints[t, l, 3].tolist() == ref.evicted, ctx
            assert delta[t, l] == ref.delta, ctx  # same fp32 operations in the same order
            np.testing.assert_allclose(weight[t, l], ref.weight, rtol=2e-6, err_msg=ctx)
            if t >= warmup:
                steady += sum(ref.miss)
        check_tables(dec, l, router, N, C)
        total += router.stats.misses
    st = dec.stats()
    assert st.misses == total and st.selections == T * L * K
    assert st.bytes_filled == total * store.blob_bytes
    print(f"replay {cfg.name} lam={lam}: {T * L} routing steps identical; misses {total} "
          f"(rate {total / (T * L * K):.5f}; after {warmup} warm-up tokens {steady / max((T - warmup) * L * K, 1):.5f}), "
          f"boundary in expert launch: {dec.plan().boundary_in_expert_launch}", flush=True)
    dec.close()
    return total


@pytest.mark.parametrize("lam", [0.5, 0.0])
def test_c2_full_shape_full_length(lam):
    """The benchmarked run itself: 24 layers x 1024 tokens at the real shape; the rate after 64 warm-up tokens is
    the figure bench.py reports at its default sizes."""
    cfg = CONFIGS["c2_qwen_bf16"]
    replay_case(cfg, lam, cfg.n_tokens, warmup=64)


@pytest.mark.parametrize("capacity", [16, 32, 48])
def test_c3_full_length_cache_sizes(capacity):
    """OLMoE shape, the three cache sizes of the cache-size ablation (Sec. 4.8)."""
    cfg = CONFIGS["c3_olmoe_bf16"].with_(inter=64, capacity=capacity)
    replay_case(cfg, 0.5, cfg.n_tokens)


def test_c4_full_length():
    cfg = CONFIGS["c4_dsv2lite_int4"].with_(inter=128, shared_inter=256)
    replay_case(cfg, 0.5, cfg.n_tokens)


def test_c5_full_length():
    cfg = CONFIGS["c5_mixtral_int8"].with_(inter=64)
    replay_case(cfg, 0.5, cfg.n_tokens)


def test_c2_prompt_phase_full_length():
    """The prompt phase at the benchmarked shape: all 24 layers, 1024 tokens in batches of 128, each layer fed its
    own exogenous stream (the batched path has no residual glue).  The device's logits of every token are replayed
    through the oracle router token by token: all decisions of all 24 x 1024 routing steps, the final tables and
    the counters are identical - a batch is its tokens in order."""
    from oracle import prompt

    cfg = CONFIGS["c2_qwen_bf16"]
    L, N, K, C, T, B = cfg.n_layers, cfg.n_experts, cfg.top_k, cfg.capacity, cfg.n_tokens, 128
    print(f"case prompt replay {cfg.name} L={L} T={T} B={B}", flush=True)
    store, dec = build(cfg, lam=0.5)
    xs = workloads.ar1_stream(cfg, T, device=DEV).to(cfg.act_dtype)
    y = torch.zeros((B, cfg.hidden), dtype=cfg.act_dtype, device=DEV)
    total = 0
    for l in range(L):
        router = routing.CachePriorRouter(N, K, C, 0.5, cfg.top_j, cfg.renormalize)
        for t0 in range(0, T, B):
            x = xs[t0:t0 + B, l].contiguous()
            recs = dec.route_batch(l, x=x)
            dec.expert_forward_batch(l, x, y)
            z = np.array([r.logits[:N] for r in recs], np.float32)
            refs = prompt.route_batch(router, z)
            for j, (r, ref) in enumerate(zip(recs, refs)):
                ctx = f"layer {l} token {t0 + j}"
                assert list(r.sel_expert[:K]) == ref.sel.tolist(), ctx
                assert list(r.sel_slot[:K]) == ref.slot and [bool(m) for m in r.miss[:K]] == ref.miss, ctx
                assert list(r.evicted[:K]) == ref.evicted and np.float32(r.delta) == ref.delta, ctx
        check_tables(dec, l, router, N, C)
        total += router.stats.misses
    st = dec.stats()
    assert st.misses == total and st.selections == T * L * K and st.bytes_filled == total * store.blob_bytes
    print(f"prompt replay: {T * L} routing steps identical, misses {total} (rate {total / (T * L * K):.5f})", flush=True)
    dec.close()
