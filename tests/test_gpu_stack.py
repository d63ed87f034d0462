"""The fused layer boundary (pending expert output + residual/normalisation glue + routing in one launch)
against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import experts as oexp
from oracle import routing, stack
from synth import workloads
from synth.workloads import CONFIGS

from _gpu_common import DEV, OracleWeights, build, route_fields

pytestmark = pytest.mark.gpu


def test_coupled_fp32_stack_fused_boundary():
    """Three coupled fp32 layers, 24 tokens: x of every layer, every routing decision and the final hidden state."""
    cfg = CONFIGS["c1_single_fp32"].with_(n_layers=3, inter=96, shared_inter=64, seed=707)
    L, K, N, d, T, lam = cfg.n_layers, cfg.top_k, cfg.n_experts, cfg.hidden, 24, 0.5
    store, dec = build(cfg, lam=lam)
    ow = OracleWeights(cfg)
    routers = [routing.CachePriorRouter(N, K, cfg.capacity, lam) for _ in range(L)]
    a = workloads.ar1_stream(cfg, T)
    a_dev = a.to(DEV)
    h = torch.zeros(d, device=DEV)
    xs = torch.zeros(L, d, device=DEV)
    y_last = torch.zeros(d, device=DEV)
    torch.cuda.synchronize()
    ties = 0
    for t in range(T):
        h_ref = a[t, 0].double().numpy()
        for l in range(L):
            raw = dec.stack_route_step(l, h, a_dev[t, l], 1.0 if l == 0 else stack.PERTURB, xs[l], carry=l > 0,
                                       y=y_last if l == 0 else None)
            dec.expert_forward(l, xs[l], None)  # output stays pending as partial rows
            dec.compute_stream.synchronize()
            out = route_fields(raw, K)
            x_ref = stack.rmsnorm(h_ref).astype(np.float32)
            assert oexp.rel_err(xs[l].cpu().numpy(), x_ref) <= 2e-6, (t, l)
            z = routing.router_logits(ow.gate(l), x_ref)
            sel, zp, delta = routers[l].select(z)
            if out["sel"] != sel.tolist():
                kth = np.sort(zp)[::-1][K - 1]
                assert np.all(zp[out["sel"]] >= kth - 1e-5), (t, l, out["sel"], sel.tolist())
                ties += 1
                sel = np.array(out["sel"])
            ref = routers[l].commit(z, sel, zp, delta)
            assert out["slot"] == ref.slot and out["miss"] == ref.miss, (t, l)
            y_ref = oexp.moe_output(x_ref, [ow.expert(l, int(e)) for e in ref.sel], ref.weight, ow.shared(l))
            if l + 1 < L:
                h_ref = stack.next_hidden(h_ref, y_ref, a[t, l + 1].numpy())
        y_prev_ref = y_ref  # the last layer's output stays pending until the next boundary call
    # flush: one more boundary call hands out the pending output of the very last layer
    dec.stack_route_step(0, h, a_dev[0, 0], 1.0, xs[0], carry=False, y=y_last)
    dec.expert_forward(0, xs[0], None)
    dec.compute_stream.synchronize()
    assert oexp.rel_err(y_last.cpu().numpy(), y_prev_ref) <= 1e-5
    for l in range(L):
        s, o = dec.stats(l), routers[l].stats
        if l > 0:
            assert (s.tokens, s.hits, s.misses) == (o.tokens, o.hits, o.misses)
    print(f"coupled fp32 stack: ties={ties}", flush=True)
    dec.close()


@pytest.mark.parametrize("name,hidden", [("c2_qwen_bf16", 2048), ("c2_qwen_bf16", 4096), ("c1_single_fp32", 256)])
def test_fused_boundary_single_step(name, hidden):
    """route + experts of layer 0 on a seeded x0, then the fused boundary of layer 1 on seeded h, a."""
    base = CONFIGS[name]
    cfg = base.with_(n_layers=2, hidden=hidden, n_experts=12, inter=128, shared_inter=128 if base.shared_inter else 0,
                     capacity=6, top_k=min(base.top_k, 4), seed=900 + hidden)
    K, N, d = cfg.top_k, cfg.n_experts, cfg.hidden
    store, dec = build(cfg, lam=0.5)
    ow = OracleWeights(cfg)
    a = workloads.ar1_stream(cfg, 3)
    x0 = a[0, 0].to(cfg.act_dtype)
    h0, a1 = a[1, 0].clone(), a[2, 1].clone()
    x0d, hd, ad = x0.to(DEV), h0.to(DEV), a1.to(DEV)
    x1d = torch.zeros(d, dtype=cfg.act_dtype, device=DEV)
    yd = torch.zeros(d, dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()
    r0 = route_fields(dec.route_step(0, x=x0d), K)
    dec.expert_forward(0, x0d, None)
    r1 = dec.stack_route_step(1, hd, ad, stack.PERTURB, x1d, carry=True, y=yd)
    dec.expert_forward(1, x1d, None)
    dec.compute_stream.synchronize()
    x0n = x0.float().numpy()
    router0 = routing.CachePriorRouter(N, K, cfg.capacity, 0.5)
    ref0 = router0.step(routing.router_logits(ow.gate(0), x0n))
    assert r0["sel"] == ref0.sel.tolist()
    y_ref = oexp.moe_output(x0n, [ow.expert(0, int(e)) for e in ref0.sel], ref0.weight, ow.shared(0))
    tol = 1e-5 if cfg.act_fmt == "fp32" else 1e-2
    assert oexp.rel_err(yd.float().cpu().numpy(), y_ref) <= tol
    y_act = torch.tensor(y_ref, dtype=torch.float32).to(cfg.act_dtype).float().numpy()  # y is an activation
    h_ref = stack.next_hidden(h0.numpy(), y_act, a1.numpy())
    assert oexp.rel_err(hd.cpu().numpy(), h_ref) <= (1e-5 if cfg.act_fmt == "fp32" else 5e-3)
    x_ref = stack.rmsnorm(h_ref)
    assert oexp.rel_err(x1d.float().cpu().numpy(), x_ref) <= (2e-6 if cfg.act_fmt == "fp32" else 2.0 ** -7)
    # routing of layer 1: the logits the device used must match the oracle's up to the rounding of x
    z_ref = routing.router_logits(ow.gate(1), torch.tensor(x_ref).to(cfg.act_dtype).float().numpy())
    z_gpu = np.array(r1.logits[:N], np.float32)
    assert np.abs(z_gpu - z_ref).max() <= (1e-5 if cfg.act_fmt == "fp32" else 3e-2) * np.abs(z_ref).max()
    sel_gpu = list(r1.sel_expert[:K])
    assert sorted(sel_gpu) == sorted(routing.ranking(z_gpu)[:K].tolist())  # empty cache: plain top-K of its own logits
    dec.close()


def run_in_launch_boundary(cfg, T, lam, outputs_every=1, force=True, monkeypatch=None):
    """A coupled stack driven as bench.py drives it - no host waiting for the decision, so that the boundary runs
    in workgroup 0 of the layer's expert launch (reduce_glue_kernel + one expert launch per layer).  Every
    layer-token is checked against the oracle fed with the device's own inputs of that step (its h before the
    step, the y it was handed, its x): h, x, logits, the routing decision incl. slots and misses (tie protocol),
    and, for every outputs_every-th step, y one step later.  Returns (ties, misses)."""
    L, K, N, d = cfg.n_layers, cfg.top_k, cfg.n_experts, cfg.hidden
    if force:
        monkeypatch.setenv("MOE_FUSE_BOUNDARY", "1")  # also without a shared expert (read when the context is created)
    store, dec = build(cfg, lam=lam)
    ow = OracleWeights(cfg)
    routers = [routing.CachePriorRouter(N, K, cfg.capacity, lam, 0, cfg.renormalize) for _ in range(L)]
    a = workloads.ar1_stream(cfg, T)
    a_dev = a.to(DEV)
    h = torch.zeros(d, device=DEV)
    x = torch.zeros(d, dtype=cfg.act_dtype, device=DEV)
    y = torch.zeros(d, dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()
    assert dec.plan().boundary_in_expert_launch == 1
    ties = misses = step = 0
    y_ref_prev = None  # oracle output of the previous layer-token, from the device's x of that step
    for t in range(T):
        for l in range(L):
            print(f"case in-launch boundary {cfg.name} d={d} token {t} layer {l}", flush=True)
            h_before = h.cpu().numpy().astype(np.float64)
            perturb = 1.0 if l == 0 else stack.PERTURB
            assert dec.stack_route_step(l, h, a_dev[t, l], perturb, x, carry=l > 0, y=y, wait=False) is None
            dec.expert_forward(l, x, None)
            raw = dec.last_route(l)
            dec.compute_stream.synchronize()
            out = route_fields(raw, K)
            ctx = (t, l)
            # y handed out by this boundary = output of the previous layer-token
            if y_ref_prev is not None:
                assert oexp.rel_err(y.float().cpu().numpy(), y_ref_prev) <= 1e-2, ctx
            y_dev = y.float().cpu().numpy().astype(np.float64)
            a_np = a[t, l].double().numpy()
            h_ref = perturb * a_np if l == 0 else stack.next_hidden(h_before, y_dev, a[t, l].numpy())
            assert oexp.rel_err(h.cpu().numpy(), h_ref) <= 1e-5, ctx
            x_ref = stack.rmsnorm(h.cpu().numpy().astype(np.float64))
            x_np = x.float().cpu().numpy()
            assert oexp.rel_err(x_np, x_ref) <= 2.0 ** -7, ctx
            z = routing.router_logits(ow.gate(l), x_np)
            z_gpu = np.array(raw.logits[:N], np.float32)
            assert np.abs(z_gpu - z).max() <= 1e-4 * max(np.abs(z).max(), 1e-3), ctx
            sel, zp, delta = routers[l].select(z)
            if out["sel"] != sel.tolist():
                kth = np.sort(zp)[::-1][K - 1]
                forced = {int(e) for e in np.nonzero(zp > kth + 1e-5)[0]}
                assert np.all(zp[out["sel"]] >= kth - 1e-5) and forced <= set(out["sel"]), (ctx, out["sel"], sel.tolist())
                ties += 1
                sel = np.array(out["sel"])
            ref = routers[l].commit(z, sel, zp, delta)
            assert out["slot"] == ref.slot and out["miss"] == ref.miss and out["evicted"] == ref.evicted, ctx
            misses += sum(ref.miss)
            y_ref_prev = None
            if step % outputs_every == 0:
                y_ref_prev = oexp.moe_output(x_np, [ow.expert(l, int(e)) for e in ref.sel], ref.weight, ow.shared(l))
            step += 1
    for l in range(L):
        s, o = dec.stats(l), routers[l].stats
        assert (s.tokens, s.hits, s.misses, s.evictions) == (o.tokens, o.hits, o.misses, o.evictions)
    print(f"in-launch boundary {cfg.name} d={d}: ties={ties} misses={misses}", flush=True)
    dec.close()
    return ties, misses


@pytest.mark.parametrize("name,hidden,inter", [("c2_qwen_bf16", 2048, 96), ("c2_qwen_bf16", 1024, 64),
                                               ("c2_qwen_bf16", 512, 64), ("c4_dsv2lite_int4", 2048, 128),
                                               ("c4_dsv2lite_int4", 4096, 128), ("c5_mixtral_int8", 4096, 96),
                                               ("c5_mixtral_int8", 1024, 64)])
def test_boundary_inside_the_expert_launch(name, hidden, inter, monkeypatch):
    """Reduced shapes of the three weight formats, every output checked.  Small caches force misses, so the second
    expert launch of a layer is exercised too."""
    base = CONFIGS[name]
    cfg = base.with_(n_layers=3, hidden=hidden, n_experts=12, inter=inter,
                     shared_inter=2 * inter if base.shared_inter else 0, capacity=5, top_k=min(base.top_k, 4),
                     seed=4200 + hidden + inter)
    ties, misses = run_in_launch_boundary(cfg, 16, 0.5, monkeypatch=monkeypatch)
    assert misses > cfg.top_k * cfg.n_layers  # more than the cold misses of the first token


def test_bounded_wait_error_path_and_reset(monkeypatch):
    """Failure handling of the boundary inside the expert launch, forced from the host: with a poll limit of one
    the other workgroups stop waiting before workgroup 0 has routed (no shared expert: the wait comes first).
    Every kernel still ends, the next call that names a layer reports MOE_EHIP, and a reset clears the state."""
    import paper_2412_00099_amd as pkg

    cfg = CONFIGS["c2_qwen_bf16"].with_(n_layers=1, hidden=512, n_experts=12, inter=64, shared_inter=0, capacity=5,
                                        top_k=4, seed=77)
    monkeypatch.setenv("MOE_FUSE_BOUNDARY", "1")
    monkeypatch.setenv("MOE_TAG_SPINS", "1")
    store, dec = build(cfg, lam=0.5)
    assert dec.plan().boundary_in_expert_launch == 1
    a = workloads.ar1_stream(cfg, 1).to(DEV)
    h = torch.zeros(cfg.hidden, device=DEV)
    x = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()
    print("case bounded wait: one step with a poll limit of one", flush=True)
    assert dec.stack_route_step(0, h, a[0, 0], 1.0, x, carry=False, y=None, wait=False) is None
    dec.expert_forward(0, x, None)
    dec.compute_stream.synchronize()
    with pytest.raises(pkg.MoEError) as e:
        dec.tables(0)
    assert e.value.code == pkg.MOE_EHIP
    dec.reset()
    assert dec.tables(0).count == 0 and dec.stats(0).tokens == 0
    dec.close()


def test_launch_timing_counts_and_strides():
    """moe_cache_profile: events on every n-th first-pass expert launch; only launches that covered a whole layer
    (no expert missing) are averaged."""
    cfg = CONFIGS["c2_qwen_bf16"].with_(n_layers=2, hidden=512, n_experts=8, inter=64, shared_inter=128, capacity=8,
                                        top_k=2, seed=5)
    store, dec = build(cfg, lam=0.5)
    T = 12
    a = workloads.ar1_stream(cfg, T).to(DEV)
    h = torch.zeros(cfg.hidden, device=DEV)
    x = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()

    def run():
        for t in range(T):
            for l in range(cfg.n_layers):
                dec.stack_route_step(l, h, a[t, l], 1.0 if l == 0 else stack.PERTURB, x, carry=l > 0, wait=False)
                dec.expert_forward(l, x, None)
        dec.compute_stream.synchronize()

    print("case launch timing: warm the cache (capacity = all experts)", flush=True)
    run()
    for stride, expect in ((1, T * cfg.n_layers), (5, -(-T * cfg.n_layers // 5))):
        print(f"case launch timing: stride {stride}", flush=True)
        misses_before = dec.stats().misses
        dec.profile(stride, reset=True)
        run()
        avg_us, n = dec.profile(0, reset=True)
        late_misses = dec.stats().misses - misses_before  # a launch with a (late cold) miss is timed but not counted
        assert expect - late_misses <= n <= expect and (n == expect or late_misses > 0)
        assert 0.5 < avg_us < 1000.0
    dec.profile(0, reset=True)
    run()
    assert dec.profile(0, reset=True) == (0.0, 0)
    dec.close()
