"""GPU parity of the fused router kernel against the oracle (through the C ABI).

From identical fp32 logits every decision is compared bit for bit: ranked expert ids, slots, miss flags,
evicted experts, Delta_avg, the slot table, the recency stamps and all counters.  With the router GEMV
computed on the device the logits agree to rounding; a selection that differs must be a tie below 1e-5
in the oracle's own altered logits and is logged, and the oracle then follows that branch.
"""
import numpy as np
import pytest
import torch

from oracle import routing
from synth import workloads
from synth.workloads import CONFIGS

from _gpu_common import DEV, OracleWeights, build, check_tables, route_fields

pytestmark = pytest.mark.gpu

TINY = CONFIGS["c1_single_fp32"].with_(inter=64)  # small blobs: these tests are about routing


def run_logits_case(cfg, lam, top_j, T, initial=None, scale=1.0, delta_fixed=None, logits=None, delta_per_token=False):
    store, dec = build(cfg, lam=lam, top_j=top_j, initial=initial, delta_fixed=delta_fixed,
                       delta_per_token=delta_per_token)
    N, K, C = cfg.n_experts, cfg.top_k, cfg.capacity
    routers = [routing.CachePriorRouter(N, K, C, lam, top_j, cfg.renormalize,
                                        initial[l] if initial else (), delta_fixed, delta_per_token)
               for l in range(cfg.n_layers)]
    x = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    y = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    zs = [workloads.logits_stream(cfg, T, layer=l, scale=scale) if logits is None else logits
          for l in range(cfg.n_layers)]
    zs_dev = [z.to(DEV) for z in zs]
    torch.cuda.synchronize()
    for t in range(T):
        for l in range(cfg.n_layers):
            out = route_fields(dec.route_step(l, logits=zs_dev[l][t]), K)
            dec.expert_forward(l, x, y)
            z = zs[l][t].numpy()
            ref = routers[l].step(z)
            ctx = f"token {t} layer {l}"
            assert out["sel"] == ref.sel.tolist(), ctx
            assert out["slot"] == ref.slot, ctx
            assert out["miss"] == ref.miss, ctx
            assert out["evicted"] == ref.evicted, ctx
            assert out["n_miss"] == sum(ref.miss) and out["token"] == t
            assert out["delta"] == ref.delta, ctx  # bit-exact fp32
            np.testing.assert_allclose(out["weight"], ref.weight, rtol=2e-6, err_msg=ctx)
    for l in range(cfg.n_layers):
        check_tables(dec, l, routers[l], N, C)
    st = dec.stats(-1)
    assert st.bytes_filled == st.misses * store.blob_bytes
    dec.close()
    return routers


@pytest.mark.parametrize("lam", [0.0, 0.5, 2.0])
def test_c1_routing_from_logits_bit_exact(lam):
    print(f"case c1 logits lam={lam}", flush=True)
    run_logits_case(TINY, lam, 0, 256)


@pytest.mark.parametrize("N,K,C,J,lam", [(60, 4, 30, 2, 0.5), (64, 8, 16, 0, 0.3), (64, 8, 8, 8, 1.0),
                                          (8, 2, 4, 1, 0.5), (3, 1, 1, 0, 0.7), (64, 1, 64, 0, 0.5)])
def test_shapes_and_limits_bit_exact(N, K, C, J, lam):
    print(f"case N={N} K={K} C={C} J={J} lam={lam}", flush=True)
    cfg = TINY.with_(n_experts=N, top_k=K, capacity=C, n_layers=2, seed=77 + N)
    routers = run_logits_case(cfg, lam, J, 200, scale=1.5)
    if C == N:
        assert all(r.stats.misses == r.stats.cold_misses for r in routers)


def test_initial_residents_renormalise_fixed_delta():
    cfg = TINY.with_(n_experts=16, top_k=2, capacity=8, n_layers=2, renormalize=True)
    init = [workloads.initial_residents(cfg, l, 8) for l in range(2)]
    print("case initial residents", flush=True)
    run_logits_case(cfg, 0.5, 1, 128, initial=init)
    print("case fixed delta", flush=True)
    run_logits_case(cfg, 0.5, 0, 64, delta_fixed=1.75)
    print("case delta = the token's own range", flush=True)
    run_logits_case(cfg, 0.5, 1, 96, delta_per_token=True, scale=1.5)


def test_fixed_points_on_device():
    cfg = TINY
    print("case huge lambda", flush=True)
    routers = run_logits_case(cfg, 1e6, 0, 128)
    assert routers[0].stats.misses == cfg.top_k  # cache freezes after the first token (Sec. 3.3)
    print("case all-equal logits", flush=True)
    z = torch.zeros(32, cfg.n_experts)
    run_logits_case(cfg, 0.5, 0, 32, logits=z)  # every ranking is a tie: index order everywhere


def test_state_errors():
    import paper_2412_00099_amd as pkg

    store, dec = build(TINY)
    x = torch.zeros(TINY.hidden, dtype=torch.float32, device=DEV)
    y = torch.zeros_like(x)
    z = torch.zeros(TINY.n_experts, dtype=torch.float32, device=DEV)
    with pytest.raises(pkg.MoEError) as e:
        dec.expert_forward(0, x, y)
    assert e.value.code == pkg.MOE_ESTATE
    dec.route_step(0, logits=z)
    with pytest.raises(pkg.MoEError) as e:
        dec.route_step(0, logits=z)
    assert e.value.code == pkg.MOE_ESTATE
    with pytest.raises(pkg.MoEError) as e:
        dec.route_step(0, x=x, logits=z)
    assert e.value.code == pkg.MOE_EINVAL
    with pytest.raises(pkg.MoEError) as e:
        dec.route_step(3, logits=z)
    assert e.value.code == pkg.MOE_EINVAL
    dec.expert_forward(0, x, y)
    dec.reset()
    assert dec.stats().tokens == 0
    dec.close()


def run_baseline_case(cfg, mode, T, top_j, max_rank=0, cumsum_p=0.0, scale=1.0):
    """Max-Rank (Eq. 6-7) and Cumsum-Threshold (Eq. 8) re-ranking on the device against the oracle's lists.

    Cumsum-Threshold turns a sum of fp32 softmax weights into the integer M: the device sums in fp32, the oracle
    in fp64, so a token whose prefix sum lies within 1e-6 of p may take either neighbouring M; both are tried and
    such tokens are logged.  Everything else is compared exactly.
    """
    import paper_2412_00099_amd as pkg
    from oracle import rerank

    route_mode = {"max_rank": pkg.MOE_ROUTE_MAX_RANK, "cumsum": pkg.MOE_ROUTE_CUMSUM}[mode]
    store, dec = build(cfg, top_j=top_j, route_mode=route_mode, max_rank=max_rank, cumsum_p=cumsum_p)
    N, K, C = cfg.n_experts, cfg.top_k, cfg.capacity
    routers = [routing.CachePriorRouter(N, K, C, 0.0, top_j, cfg.renormalize) for _ in range(cfg.n_layers)]
    x = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    y = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    zs = [workloads.logits_stream(cfg, T, layer=l, scale=scale) for l in range(cfg.n_layers)]
    zs_dev = [z.to(DEV) for z in zs]
    torch.cuda.synchronize()
    near = 0
    for t in range(T):
        for l in range(cfg.n_layers):
            out = route_fields(dec.route_step(l, logits=zs_dev[l][t]), K)
            dec.expert_forward(l, x, y)
            z = zs[l][t].numpy()
            rt = routers[l]
            delta = rt.range.update(z)
            r = routing.ranking(z).tolist()
            cache = {e for e in range(N) if rt.cache.slot_of[e] >= 0}
            ctx = f"{mode} token {t} layer {l}"
            if mode == "max_rank":
                options = [rerank.max_rank(r, cache, max_rank, top_j)[:K]]
            else:
                w = routing.softmax(z)
                prefix = np.cumsum([w[e] for e in r])
                m = rerank.cumsum_rank([w[e] for e in r], cumsum_p)
                assert m == min(int(np.searchsorted(prefix, cumsum_p, side="left")) + 1, N), ctx
                ms = {m} | {i + 1 + d for i in range(N) if abs(prefix[i] - cumsum_p) < 1e-6 for d in (0, 1) if i + 1 + d <= N}
                options = [rerank.max_rank(r, cache, mm, top_j)[:K] for mm in sorted(ms, key=lambda v: v != m)]
            if out["sel"] != options[0]:
                assert out["sel"] in options, (ctx, out["sel"], options)
                near += 1
                print(f"  {ctx}: prefix sum within 1e-6 of p, device took the neighbouring M", flush=True)
            ref = rt.commit(z, np.asarray(out["sel"]), delta=delta)
            assert out["slot"] == ref.slot and out["miss"] == ref.miss and out["evicted"] == ref.evicted, ctx
            assert out["delta"] == ref.delta and out["token"] == t, ctx
            np.testing.assert_allclose(out["weight"], ref.weight, rtol=2e-6, err_msg=ctx)
    assert near <= max(1, T * cfg.n_layers // 100)
    for l in range(cfg.n_layers):
        check_tables(dec, l, routers[l], N, C)
    dec.close()
    return routers


@pytest.mark.parametrize("M,J", [(0, 0), (8, 0), (16, 1), (60, 2), (4, 4)])
def test_max_rank_mode_bit_exact(M, J):
    print(f"case max-rank M={M} J={J}", flush=True)
    cfg = TINY.with_(n_experts=60, top_k=4, capacity=30, n_layers=2, seed=311)
    routers = run_baseline_case(cfg, "max_rank", 200, J, max_rank=M, scale=1.5)
    if M == 0 or J == cfg.top_k:
        # nothing is promoted past the router's own top-K: plain LRU caching of the original routing
        ref = [routing.CachePriorRouter(60, 4, 30, 0.0) for _ in range(2)]
        for l in range(2):
            for z in workloads.logits_stream(cfg, 200, layer=l, scale=1.5).numpy():
                ref[l].step(z)
            assert ref[l].stats.misses == routers[l].stats.misses


@pytest.mark.parametrize("p,J", [(0.0, 0), (0.3, 0), (0.7, 1), (0.95, 2), (1.5, 0)])
def test_cumsum_threshold_mode(p, J):
    print(f"case cumsum p={p} J={J}", flush=True)
    cfg = TINY.with_(n_experts=60, top_k=4, capacity=30, n_layers=2, seed=312)
    run_baseline_case(cfg, "cumsum", 200, J, cumsum_p=p, scale=1.5)


def test_snapshot_restore_resumes_bit_exactly():
    """Run, snapshot, run on; then reset, restore and run the same tokens again: same decisions, same outputs,
    same final tables (the slots are refilled from the host tier by the restore)."""
    import paper_2412_00099_amd as pkg

    cfg = TINY.with_(n_experts=16, top_k=2, capacity=6, n_layers=2, seed=91)
    store, dec = build(cfg, lam=0.3)
    N, K = cfg.n_experts, cfg.top_k
    T1, T2 = 40, 40
    zs = [workloads.logits_stream(cfg, T1 + T2, layer=l, scale=1.5).to(DEV) for l in range(cfg.n_layers)]
    xs = workloads.ar1_stream(cfg, T1 + T2, device=DEV)[:, 0].to(cfg.act_dtype)
    y = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)

    def run(t0, t1):
        rec = []
        for t in range(t0, t1):
            for l in range(cfg.n_layers):
                out = route_fields(dec.route_step(l, logits=zs[l][t]), K)
                dec.expert_forward(l, xs[t], y)
                dec.compute_stream.synchronize()  # y.clone() runs on torch's stream, the library on its own
                rec.append((out["sel"], out["slot"], out["miss"], out["evicted"], float(out["delta"]), y.clone()))
        return rec

    print("case snapshot: first leg", flush=True)
    run(0, T1)
    snaps = [dec.snapshot(l) for l in range(cfg.n_layers)]
    stats_mid = [dec.stats(l) for l in range(cfg.n_layers)]
    first = run(T1, T1 + T2)
    tables_end = [dec.tables(l) for l in range(cfg.n_layers)]
    print("case snapshot: restore and replay", flush=True)
    dec.reset()
    for l in range(cfg.n_layers):
        dec.restore(l, snaps[l])
        s = dec.stats(l)
        assert (s.tokens, s.misses, s.evictions, s.lifetime_sum) == (
            stats_mid[l].tokens, stats_mid[l].misses, stats_mid[l].evictions, stats_mid[l].lifetime_sum)
    second = run(T1, T1 + T2)
    for a, b in zip(first, second):
        assert a[:5] == b[:5]
        assert torch.equal(a[5], b[5])
    for l in range(cfg.n_layers):
        t = dec.tables(l)
        assert list(t.expert_slot) == list(tables_end[l].expert_slot)
        assert list(t.stamp[:N]) == list(tables_end[l].stamp[:N])
    # a damaged blob is refused and changes nothing
    bad = bytearray(snaps[0])
    bad[24] ^= 0x7f  # first table entry
    with pytest.raises(pkg.MoEError) as e:
        dec.restore(0, bytes(bad))
    assert e.value.code == pkg.MOE_EINVAL
    with pytest.raises(pkg.MoEError):
        dec.restore(0, snaps[0][:100])
    assert list(dec.tables(0).expert_slot) == list(tables_end[0].expert_slot)
    dec.close()


def test_device_trace_lru_and_optimal_eviction_bound():
    """Record the original routing (lambda = 0) on the device, then replay the trace through the library's offline
    simulator and the oracle's: the device's own miss count equals the simulated LRU count at the same capacity,
    farthest-next-use eviction (Sec. 4.8) is never worse, and both agree with the oracle at every cache size."""
    import paper_2412_00099_amd as pkg
    from oracle import eviction

    cfg = TINY.with_(n_experts=24, top_k=3, capacity=8, n_layers=1, seed=17)
    store, dec = build(cfg, lam=0.0)
    N, K, C = cfg.n_experts, cfg.top_k, cfg.capacity
    T = 300
    zs = workloads.logits_stream(cfg, T, layer=0, scale=1.5)
    zs_dev = zs.to(DEV)
    x = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    y = torch.zeros_like(x)
    trace = np.zeros((T, K), np.int32)
    print("case device trace", flush=True)
    for t in range(T):
        out = dec.route_step(0, logits=zs_dev[t])
        dec.expert_forward(0, x, y)
        trace[t] = list(out.sel_expert[:K])  # at lambda = 0 the ranking by z' is the touch order
    st = dec.stats(0)
    dec.close()
    lru, life, ev = pkg.moe_trace_misses(trace, N, C, pkg.MOE_POLICY_LRU)
    assert (lru, life, ev) == (st.misses, st.lifetime_sum, st.evictions)
    opt, _, _ = pkg.moe_trace_misses(trace, N, C, pkg.MOE_POLICY_FARTHEST)
    assert opt <= lru and opt == eviction.belady_misses(trace.tolist(), C)
    prev = None
    for c in range(1, N + 1):
        m, _, _ = pkg.moe_trace_misses(trace, N, c, pkg.MOE_POLICY_LRU)
        assert m == eviction.lru_list_misses(trace.tolist(), c)[0]
        assert prev is None or m <= prev  # LRU is a stack algorithm per token set: more slots never hurt
        prev = m
    assert prev == len(set(trace.ravel().tolist()))  # cache of all experts: only first touches miss


def free_run(cfg, lam, T, top_j=0, check_outputs_every=1, tol=None, deferred=False):
    """x-in mode: the device computes the router GEMV; tie protocol on disagreement."""
    from oracle import experts as oexp

    tol = tol or (1e-5 if cfg.act_fmt == "fp32" else 1e-2)
    store, dec = build(cfg, lam=lam, top_j=top_j)
    N, K, C, L = cfg.n_experts, cfg.top_k, cfg.capacity, cfg.n_layers
    ow = OracleWeights(cfg)
    routers = [routing.CachePriorRouter(N, K, C, lam, top_j, cfg.renormalize) for _ in range(L)]
    a = workloads.ar1_stream(cfg, T)  # [T, L, d] fp32, exogenous input of every layer
    xs = a.to(cfg.act_dtype)
    xs_dev = xs.to(DEV)
    ys = torch.zeros((T, L, cfg.hidden), dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()
    ties, worst_y, worst_z = 0, 0.0, 0.0
    picks = []
    for t in range(T):
        for l in range(L):
            if deferred:  # the router kernel is only enqueued; the decision is collected by expert_forward
                assert dec.route_step(l, x=xs_dev[t, l], wait=False) is None
                dec.expert_forward(l, xs_dev[t, l], ys[t, l])
                raw = dec.last_route(l)
            else:
                raw = dec.route_step(l, x=xs_dev[t, l])
                dec.expert_forward(l, xs_dev[t, l], ys[t, l])
            out = route_fields(raw, K)
            x_np = xs[t, l].float().numpy()
            z = routing.router_logits(ow.gate(l), x_np)
            z_gpu = np.array(raw.logits[:N], np.float32)
            worst_z = max(worst_z, float(np.abs(z_gpu - z).max() / np.abs(z).max()))
            sel, zp, delta = routers[l].select(z)
            ctx = f"token {t} layer {l}"
            if out["sel"] != sel.tolist():
                kth = np.sort(zp)[::-1][K - 1]
                chosen = zp[out["sel"]]
                forced = {int(e) for e in np.nonzero(zp > kth + 1e-5)[0]}
                assert np.all(chosen >= kth - 1e-5) and forced <= set(out["sel"]), (
                    f"{ctx}: device {out['sel']} vs oracle {sel.tolist()} is not a tie "
                    f"(margin {routing.topk_margin(zp, K):.3g})")
                ties += 1
                print(f"tie logged at {ctx}: margin {routing.topk_margin(zp, K):.3g}", flush=True)
                sel = np.array(out["sel"])
            ref = routers[l].commit(z, sel, zp, delta)
            assert out["slot"] == ref.slot and out["miss"] == ref.miss and out["evicted"] == ref.evicted, ctx
            assert abs(float(out["delta"]) - float(ref.delta)) <= 1e-5 * float(ref.delta), ctx
            np.testing.assert_allclose(out["weight"], ref.weight, rtol=1e-4 if cfg.act_fmt == "fp32" else 1e-2)
            picks.append((t, l, x_np, ref))
    dec.compute_stream.synchronize()
    ys_np = ys.float().cpu().numpy()
    for i, (t, l, x_np, ref) in enumerate(picks):
        if i % check_outputs_every:
            continue
        y_ref = oexp.moe_output(x_np, [ow.expert(l, int(e)) for e in ref.sel], ref.weight, ow.shared(l))
        err = oexp.rel_err(ys_np[t, l], y_ref)
        worst_y = max(worst_y, err)
        assert err <= tol, f"token {t} layer {l}: rel err {err:.3g} > {tol}"
    for l in range(L):
        s, o = dec.stats(l), routers[l].stats
        assert (s.tokens, s.hits, s.misses, s.cold_misses, s.evictions) == (
            o.tokens, o.hits, o.misses, o.cold_misses, o.evictions)
    assert worst_z <= (1e-5 if cfg.act_fmt == "fp32" else 1e-4)
    print(f"{cfg.name} lam={lam}: ties={ties} worst logit err={worst_z:.3g} worst output err={worst_y:.3g} "
          f"miss rate={dec.stats().misses / max(dec.stats().selections, 1):.3f}", flush=True)
    dec.close()
    return ties


@pytest.mark.parametrize("lam", [0.0, 0.5, 2.0])
def test_c1_free_run_routing_and_outputs(lam):
    print(f"case c1 free run lam={lam}", flush=True)
    free_run(CONFIGS["c1_single_fp32"], lam, 256)


@pytest.mark.parametrize("lam", [0.0, 0.5])
def test_c1_free_run_deferred_decision(lam):
    print(f"case c1 deferred lam={lam}", flush=True)
    free_run(CONFIGS["c1_single_fp32"], lam, 128, deferred=True)


@pytest.mark.parametrize("h", [2, 3, 4, 5])
def test_pruning_baseline_on_device(h):
    """Pruning baseline (Sec. 4.2): of the router's top-K the experts ranked >= h (ranks from 1) are discarded; on
    the device that is the original routing (lambda = 0) with h - 1 experts per token.  Selections, slots, misses and
    evictions against oracle.rerank.prune fed through the oracle cache; the miss rate is normalised by the
    original K on both sides."""
    from oracle import rerank

    K = 4
    cfg = TINY.with_(n_experts=60, top_k=min(K, h - 1), capacity=30, n_layers=1, seed=313)
    print(f"case pruning h={h} (keeps {cfg.top_k} of {K})", flush=True)
    store, dec = build(cfg, lam=0.0)
    N, C, T = cfg.n_experts, cfg.capacity, 300
    cache = routing.ExpertCache(N, C)
    x = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    y = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    zs = workloads.logits_stream(cfg, T, layer=0, scale=1.5)
    zs_dev = zs.to(DEV)
    torch.cuda.synchronize()
    for t in range(T):
        out = route_fields(dec.route_step(0, logits=zs_dev[t]), cfg.top_k)
        dec.expert_forward(0, x, y)
        z = zs[t].numpy()
        kept = rerank.prune(routing.ranking(z).tolist(), K, h)
        miss, slot, evicted = cache.access(kept, z)
        assert out["sel"] == kept and out["slot"] == slot and out["miss"] == miss and out["evicted"] == evicted, t
        np.testing.assert_allclose(out["weight"], routing.softmax(z)[kept], rtol=2e-6)
    st = dec.stats(0)
    assert (st.misses, st.evictions, st.lifetime_sum) == (cache.stats.misses, cache.stats.evictions,
                                                          cache.stats.lifetime_sum)
    assert rerank.pruned_miss_rate(st.misses, T, K) == rerank.pruned_miss_rate(cache.stats.misses, T, K) <= (h - 1) / K
    if h == K + 1:  # nothing pruned: the original routing with plain LRU
        ref = routing.CachePriorRouter(N, K, C, 0.0)
        for z in zs.numpy():
            ref.step(z)
        assert ref.stats.misses == st.misses
    dec.close()
