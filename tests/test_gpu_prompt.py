"""Prompt phase (a batch of tokens through a layer) against the oracle, through the C ABI.

Routing from identical fp32 logits must equal the oracle's token-by-token routing bit for bit - and therefore what
the single-token entry point does.  With the gate logits computed on the device (matrix cores) the tie protocol of
the other tests applies.  Outputs are compared per token to the output tolerance; the per-expert tiles of a token
are added in a fixed order, so two runs give identical bits."""
import numpy as np
import pytest
import torch

from oracle import experts as oexp
from oracle import prompt, routing
from synth import workloads
from synth.workloads import CONFIGS

from _gpu_common import DEV, OracleWeights, build, check_tables, route_fields

pytestmark = pytest.mark.gpu

BASE = CONFIGS["c2_qwen_bf16"]


@pytest.mark.parametrize("batches,N,K,C,J,lam", [([8, 32, 128, 1, 37], 60, 4, 30, 0, 0.5), ([128, 128], 64, 8, 16, 2, 0.3),
                                                 ([5, 64], 8, 2, 2, 0, 0.5)])
def test_batch_routing_from_logits_bit_exact(batches, N, K, C, J, lam):
    cfg = BASE.with_(n_layers=2, hidden=1024, n_experts=N, inter=32, shared_inter=32, top_k=K, capacity=C, seed=610 + N)
    print(f"case prompt routing N={N} K={K} C={C} J={J} batches={batches}", flush=True)
    store, dec = build(cfg, lam=lam, top_j=J)
    T = sum(batches)
    routers = [routing.CachePriorRouter(N, K, C, lam, J) for _ in range(cfg.n_layers)]
    x = torch.zeros((max(batches), cfg.hidden), dtype=cfg.act_dtype, device=DEV)
    y = torch.zeros_like(x)
    for l in range(cfg.n_layers):
        zs = workloads.logits_stream(cfg, T, layer=l, scale=1.5)
        zs_dev = zs.to(DEV)
        t0 = 0
        for i, b in enumerate(batches):
            if i == 1:  # a single-token step in between: both entry points walk the same state
                out = route_fields(dec.route_step(l, logits=zs_dev[t0]), K)
                dec.expert_forward(l, x[0], y[0])
                ref = routers[l].step(zs[t0].numpy())
                assert out["sel"] == ref.sel.tolist() and out["slot"] == ref.slot and out["miss"] == ref.miss
                t0 += 1
                b -= 1
                if b == 0:
                    continue
            recs = dec.route_batch(l, logits=zs_dev[t0:t0 + b].contiguous())
            dec.expert_forward_batch(l, x[:b], y[:b])
            refs = prompt.route_batch(routers[l], zs[t0:t0 + b].numpy())
            for j, (raw, ref) in enumerate(zip(recs, refs)):
                out = route_fields(raw, K)
                ctx = f"layer {l} batch {i} token {j}"
                assert out["sel"] == ref.sel.tolist(), ctx
                assert out["slot"] == ref.slot and out["miss"] == ref.miss and out["evicted"] == ref.evicted, ctx
                assert out["delta"] == ref.delta and out["token"] == t0 + j, ctx
                np.testing.assert_allclose(out["weight"], ref.weight, rtol=2e-6, err_msg=ctx)
            t0 += b
        check_tables(dec, l, routers[l], N, C)
    st = dec.stats()
    assert st.bytes_filled == st.misses * store.blob_bytes
    dec.close()


def run_prompt_outputs(cfg, lam, batches, every=1):
    store, dec = build(cfg, lam=lam)
    N, K, C, d = cfg.n_experts, cfg.top_k, cfg.capacity, cfg.hidden
    ow = OracleWeights(cfg)
    router = routing.CachePriorRouter(N, K, C, lam, 0, cfg.renormalize)
    T = sum(batches)
    xs = workloads.ar1_stream(cfg, T)[:, 0].to(cfg.act_dtype)
    xs_dev = xs.to(DEV)
    ys = torch.zeros((T, d), dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()
    t0, ties, worst, worst_z = 0, 0, 0.0, 0.0
    for b in batches:
        print(f"case prompt outputs {cfg.name} d={d} I={cfg.inter} B={b} tokens {t0}..{t0 + b - 1}", flush=True)
        recs = dec.route_batch(0, x=xs_dev[t0:t0 + b])
        dec.expert_forward_batch(0, xs_dev[t0:t0 + b], ys[t0:t0 + b])
        y_np = ys[t0:t0 + b].float().cpu().numpy()
        for j, raw in enumerate(recs):
            out = route_fields(raw, K)
            x_np = xs[t0 + j].float().numpy()
            z = routing.router_logits(ow.gate(0), x_np)
            z_gpu = np.array(raw.logits[:N], np.float32)
            worst_z = max(worst_z, float(np.abs(z_gpu - z).max() / np.abs(z).max()))
            sel, zp, delta = router.select(z)
            ctx = f"token {t0 + j}"
            if out["sel"] != sel.tolist():
                kth = np.sort(zp)[::-1][K - 1]
                forced = {int(e) for e in np.nonzero(zp > kth + 1e-5)[0]}
                assert np.all(zp[out["sel"]] >= kth - 1e-5) and forced <= set(out["sel"]), (ctx, out["sel"], sel.tolist())
                ties += 1
                sel = np.array(out["sel"])
            ref = router.commit(z, sel, zp, delta)
            assert out["slot"] == ref.slot and out["miss"] == ref.miss and out["evicted"] == ref.evicted, ctx
            if (t0 + j) % every == 0:
                y_ref = oexp.moe_output(x_np, [ow.expert(0, int(e)) for e in ref.sel], ref.weight, ow.shared(0))
                err = oexp.rel_err(y_np[j], y_ref)
                worst = max(worst, err)
                assert err <= 1e-2, f"{ctx}: rel err {err:.3g}"
        t0 += b
    s, o = dec.stats(0), router.stats
    assert (s.tokens, s.hits, s.misses, s.cold_misses, s.evictions, s.lifetime_sum) == (
        o.tokens, o.hits, o.misses, o.cold_misses, o.evictions, o.lifetime_sum)
    assert worst_z <= 1e-4
    print(f"prompt {cfg.name}: ties={ties} worst logit err={worst_z:.3g} worst output err={worst:.3g} "
          f"misses={s.misses}/{s.selections}", flush=True)
    dec.close()


@pytest.mark.parametrize("hidden,inter,shared,N,K,C,lam", [(2048, 160, 320, 12, 4, 5, 0.5), (1024, 48, 0, 10, 2, 3, 0.0),
                                                           (2048, 272, 144, 60, 4, 30, 0.25), (2048, 64, 64, 12, 4, 4, 0.0)])
def test_batch_outputs_reduced_shapes(hidden, inter, shared, N, K, C, lam):
    """Small caches: slots are refilled inside a batch, so batches are cut into several expert launches; ragged
    batch sizes, a batch of one, tiles of more and fewer than 16 tokens per expert."""
    cfg = BASE.with_(n_layers=1, hidden=hidden, n_experts=N, inter=inter, shared_inter=shared, top_k=K, capacity=C,
                     seed=7000 + inter)
    run_prompt_outputs(cfg, lam, [8, 37, 1, 128, 16])


def test_batch_outputs_full_layer_shape():
    """The benchmarked layer shape (60 experts of 1408, shared 5632, cache 30), batches of 32 and 128; outputs of
    every 9th token against the oracle."""
    cfg = BASE.with_(n_layers=1)
    run_prompt_outputs(cfg, 0.5, [32, 128], every=9)


def test_batch_outputs_olmoe_layer_shape():
    """The OLMoE-shaped layer (64 experts of 1024, no shared expert, top-8, cache 32): batches of 128, 16 and 40;
    outputs of every 11th token against the oracle."""
    cfg = CONFIGS["c3_olmoe_bf16"].with_(n_layers=1)
    run_prompt_outputs(cfg, 0.5, [128, 16, 40], every=11)


def test_batch_outputs_are_reproducible():
    cfg = BASE.with_(n_layers=1, hidden=2048, n_experts=16, inter=96, shared_inter=160, top_k=4, capacity=6, seed=616)
    store, dec = build(cfg, lam=0.25)
    xs = workloads.ar1_stream(cfg, 100)[:, 0].to(cfg.act_dtype).to(DEV)
    outs = []
    for rep in range(2):
        dec.reset()
        y = torch.zeros((100, cfg.hidden), dtype=cfg.act_dtype, device=DEV)
        for t0, b in ((0, 36), (36, 64)):
            dec.route_batch(0, x=xs[t0:t0 + b])
            dec.expert_forward_batch(0, xs[t0:t0 + b], y[t0:t0 + b])
        outs.append(y)
    assert torch.equal(outs[0], outs[1])
    dec.close()


def test_batch_equals_single_token_path_and_errors():
    """The same tokens through the single-token entry points: identical decisions and counters, outputs equal to
    rounding; then the error paths."""
    import paper_2412_00099_amd as pkg

    cfg = BASE.with_(n_layers=1, hidden=1024, n_experts=16, inter=64, shared_inter=64, top_k=2, capacity=6, seed=615)
    store, dec = build(cfg, lam=0.5)
    store2, dec2 = build(cfg, lam=0.5)
    B = 48
    xs = workloads.ar1_stream(cfg, B)[:, 0].to(cfg.act_dtype).to(DEV)
    yb = torch.zeros((B, cfg.hidden), dtype=cfg.act_dtype, device=DEV)
    y1 = torch.zeros_like(yb)
    recs = dec.route_batch(0, x=xs)
    dec.expert_forward_batch(0, xs, yb)
    singles = []
    for t in range(B):
        singles.append(dec2.route_step(0, x=xs[t]))
        dec2.expert_forward(0, xs[t], y1[t])
    dec2.compute_stream.synchronize()
    for a, b in zip(recs, singles):
        fa, fb = route_fields(a, cfg.top_k), route_fields(b, cfg.top_k)
        # the two gate products differ in summation order: same decisions unless a top-K margin is below 1e-5
        assert fa["sel"] == fb["sel"] or min(a.margin, b.margin) < 1e-5
    if all(route_fields(a, 2)["sel"] == route_fields(b, 2)["sel"] for a, b in zip(recs, singles)):
        sa, sb = dec.stats(0), dec2.stats(0)
        assert (sa.misses, sa.evictions, sa.lifetime_sum) == (sb.misses, sb.evictions, sb.lifetime_sum)
        assert oexp.rel_err(yb.float().cpu().numpy(), y1.float().cpu().numpy()) <= 1e-2
    # error paths
    with pytest.raises(pkg.MoEError) as e:
        dec.expert_forward_batch(0, xs, yb)  # no routed batch pending
    assert e.value.code == pkg.MOE_ESTATE
    dec.route_batch(0, x=xs[:4])
    with pytest.raises(pkg.MoEError) as e:
        dec.route_step(0, x=xs[0])  # a batch is pending
    assert e.value.code == pkg.MOE_ESTATE
    with pytest.raises(pkg.MoEError) as e:
        dec.expert_forward_batch(0, xs[:5], yb[:5])  # wrong size
    assert e.value.code == pkg.MOE_ESTATE
    dec.expert_forward_batch(0, xs[:4], yb[:4])
    with pytest.raises(pkg.MoEError) as e:
        pkg.moe_route_batch(dec.ctx, 0, None, None, 4)
    assert e.value.code == pkg.MOE_EINVAL
    dec.close()
    dec2.close()
    # shapes the batched kernels do not take are refused, not computed some other way
    c1 = CONFIGS["c1_single_fp32"].with_(inter=64)
    store3, dec3 = build(c1, lam=0.5)
    z = torch.zeros((4, c1.n_experts), device=DEV)
    with pytest.raises(pkg.MoEError) as e:
        dec3.route_batch(0, logits=z)
    assert e.value.code == pkg.MOE_EINVAL
    dec3.close()


@pytest.mark.parametrize("mode", ["lru", "strong_prior", "max_rank", "cumsum", "delta_fixed", "delta_token", "renorm_topj",
                                  "initial_residents"])
@pytest.mark.parametrize("C", [3, 12])
def test_batch_routing_equals_token_by_token_in_every_mode(mode, C):
    """The batch routing accepts the tokens of a window up to the first miss and routes the missing token alone:
    in every routing mode, with frequent (C = 3) and rare (C = 12) misses, its records, tables and counters must be
    those of the single-token steps (which the routing tests hold against the oracle), bit for bit."""
    import paper_2412_00099_amd as pkg

    kw = dict(lru=dict(lam=0.0), strong_prior=dict(lam=2.0), max_rank=dict(route_mode=pkg.MOE_ROUTE_MAX_RANK, max_rank=8, top_j=1),
              cumsum=dict(route_mode=pkg.MOE_ROUTE_CUMSUM, cumsum_p=0.7), delta_fixed=dict(lam=0.5, delta_fixed=1.25),
              delta_token=dict(lam=0.7, delta_per_token=True), renorm_topj=dict(lam=0.5, top_j=1),
              initial_residents=dict(lam=0.5, initial=[[5, 2, 9][:min(C, 3)]]))[mode]
    N, K = 16, 3
    cfg = BASE.with_(n_layers=1, hidden=1024, n_experts=N, inter=32, shared_inter=32, top_k=K, capacity=C,
                     renormalize=mode == "renorm_topj", seed=930 + C)
    print(f"case batch routing vs single tokens: {mode} C={C}", flush=True)
    store_a, one = build(cfg, **kw)
    store_b, many = build(cfg, **kw)
    batches = [128, 1, 37, 16, 17, 128, 5]
    T = sum(batches)
    zs = workloads.logits_stream(cfg, T, layer=0, scale=1.5).to(DEV)
    x = torch.zeros((128, cfg.hidden), dtype=cfg.act_dtype, device=DEV)
    y = torch.zeros_like(x)
    t0 = 0
    for b in batches:
        recs = many.route_batch(0, logits=zs[t0:t0 + b].contiguous())
        many.expert_forward_batch(0, x[:b], y[:b])
        for j in range(b):
            ref = one.route_step(0, logits=zs[t0 + j])
            one.expert_forward(0, x[0], y[0])
            fa, fb = route_fields(ref, K), route_fields(recs[j], K)
            for key in fa:
                assert np.array_equal(fa[key], fb[key]), (t0 + j, key, fa[key], fb[key])
            assert list(ref.logits[:N]) == list(recs[j].logits[:N])
        t0 += b
    ta, tb = one.tables(0), many.tables(0)
    for field in ("expert_slot", "slot_expert", "stamp"):
        assert list(getattr(ta, field)) == list(getattr(tb, field)), field
    assert (ta.count, ta.delta_sum) == (tb.count, tb.delta_sum)
    sa, sb = one.stats(0), many.stats(0)
    for field in ("tokens", "selections", "hits", "misses", "cold_misses", "evictions", "lifetime_sum", "bytes_filled"):
        assert getattr(sa, field) == getattr(sb, field), field
    assert sa.misses >= K and (mode != "lru" or C != 3 or sa.misses > T // 4)
    one.close()
    many.close()
