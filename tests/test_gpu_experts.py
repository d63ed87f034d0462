"""GPU parity of the expert SwiGLU GEMV (and the packer) against the oracle, through the C ABI.

Tolerance (max_j |y - y_ref| / max_j |y_ref|): 1e-5 for fp32 weights and activations, 1e-2 for bf16
activations with fp32 accumulation.
"""
import math

import numpy as np
import pytest
import torch

from oracle import experts as oexp
from oracle import stack as ostack
from synth.workloads import CONFIGS

from _gpu_common import DEV, build
from test_gpu_route import free_run

pytestmark = pytest.mark.gpu

C1 = CONFIGS["c1_single_fp32"]
C2 = CONFIGS["c2_qwen_bf16"]


@pytest.mark.parametrize("deferred", [False, True])
def test_bf16_stack_reduced_with_shared_expert_and_ragged_split(deferred):
    # 4*200 + 328 = 1128 records over 256 workgroups of 8 wavefronts: uneven spans, idle wavefronts;
    # lambda = 0 keeps misses frequent, so the second (post-fill) expert launch is exercised often
    cfg = C2.with_(n_layers=2, n_experts=12, inter=200, shared_inter=328, capacity=6, seed=91)
    print(f"case bf16 reduced stack deferred={deferred}", flush=True)
    free_run(cfg, 0.5, 48, top_j=2, deferred=deferred)
    free_run(cfg, 0.0, 48, deferred=deferred)


@pytest.mark.parametrize("fmt,hidden", [("fp32", 512), ("fp32", 1024), ("fp32", 2048), ("bf16", 512),
                                        ("bf16", 1024), ("bf16", 4096)])
def test_other_hidden_sizes(fmt, hidden):
    cfg = C1.with_(hidden=hidden, inter=96, shared_inter=40, n_experts=8, capacity=4, weight_fmt=fmt, act_fmt=fmt,
                   seed=300 + hidden)
    print(f"case {fmt} hidden={hidden}", flush=True)
    free_run(cfg, 0.5, 24)


def test_fewer_records_than_wavefronts():
    cfg = C1.with_(inter=3, n_experts=4, capacity=2, seed=5)
    print("case tiny inter", flush=True)
    free_run(cfg, 0.0, 16)


def test_top8_of_64_olmoe_like_reduced():
    cfg = CONFIGS["c3_olmoe_bf16"].with_(n_layers=1, inter=64, capacity=16, seed=8)
    print("case olmoe reduced", flush=True)
    free_run(cfg, 0.5, 32)


def test_mixtral_like_renormalised_reduced():
    cfg = CONFIGS["c5_mixtral_int8"].with_(n_layers=2, inter=160, weight_fmt="bf16", seed=9)
    print("case mixtral-shaped bf16 reduced", flush=True)
    free_run(cfg, 0.5, 32, top_j=1)


def test_packer_layout_closed_form():
    """One non-zero per matrix: y = down[j3,i] * silu(gate[i,j1]*x[j1]) * up[i,j2]*x[j2] * w lands on output j3 only."""
    cfg = C1.with_(n_experts=2, capacity=2, top_k=1, inter=40)
    store, dec = build(cfg)
    d, I = cfg.hidden, cfg.inter
    i, j1, j2, j3 = 37, 3, 200, 129
    g = torch.zeros(I, d); u = torch.zeros(I, d); dn = torch.zeros(d, I)
    g[i, j1], u[i, j2], dn[j3, i] = 2.0, -1.5, 4.0
    store.put_expert(0, 1, {"gate": g, "up": u, "down": dn})
    x = torch.zeros(d); x[j1], x[j2] = 0.75, 2.0
    xd, yd = x.to(DEV), torch.zeros(d, device=DEV)
    z = torch.tensor([0.0, 5.0], device=DEV)
    torch.cuda.synchronize()
    out = dec.route_step(0, logits=z)
    assert list(out.sel_expert[:1]) == [1]
    dec.expert_forward(0, xd, yd)
    dec.compute_stream.synchronize()
    a = 2.0 * 0.75
    w = math.exp(5.0) / (1.0 + math.exp(5.0))
    expect = 4.0 * (a / (1 + math.exp(-a))) * (-1.5 * 2.0) * w
    y = yd.cpu().numpy()
    assert abs(y[j3] - expect) <= 1e-5 * abs(expect)
    y[j3] = 0
    assert np.all(y == 0)
    dec.close()


@pytest.mark.parametrize("fmt", ["fp32", "bf16"])
def test_stack_glue_kernel(fmt):
    import paper_2412_00099_amd as pkg

    cfg = C2.with_(n_layers=1, n_experts=4, inter=8, shared_inter=0, capacity=4, weight_fmt=fmt, act_fmt=fmt)
    store, dec = build(cfg)
    d = cfg.hidden
    g = torch.Generator().manual_seed(4)
    h = torch.randn(d, generator=g)
    y = (torch.randn(d, generator=g) * 0.3).to(cfg.act_dtype)
    a = torch.randn(d, generator=g)
    hd, yd, ad = h.to(DEV), y.to(DEV), a.to(DEV)
    xd = torch.zeros(d, dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()
    dec.residual_rmsnorm(hd, yd, ad, ostack.PERTURB, xd)
    dec.compute_stream.synchronize()
    h_ref = ostack.next_hidden(h.numpy(), y.float().numpy(), a.numpy())
    x_ref = ostack.rmsnorm(h_ref)
    assert oexp.rel_err(hd.cpu().numpy(), h_ref) <= 1e-6
    assert oexp.rel_err(xd.float().cpu().numpy(), x_ref) <= (1e-6 if fmt == "fp32" else 4e-3)
    dec.close()


# ---------------------------------------------------------------- weight-only int8 / int4


@pytest.mark.parametrize("hidden,inter", [(4096, 160), (2048, 104), (1024, 64)])
def test_int8_reduced(hidden, inter):
    cfg = CONFIGS["c5_mixtral_int8"].with_(n_layers=2, hidden=hidden, inter=inter, seed=400 + hidden)
    print(f"case int8 hidden={hidden}", flush=True)
    free_run(cfg, 0.5, 32, top_j=1)
    free_run(cfg, 0.0, 24, deferred=True)


@pytest.mark.parametrize("hidden,inter,shared", [(2048, 256, 384), (4096, 128, 0)])
def test_int4_reduced(hidden, inter, shared):
    cfg = CONFIGS["c4_dsv2lite_int4"].with_(n_layers=2, hidden=hidden, inter=inter, shared_inter=shared,
                                            n_experts=16, capacity=8, seed=500 + hidden)
    print(f"case int4 hidden={hidden}", flush=True)
    free_run(cfg, 0.5, 32, top_j=2)
    free_run(cfg, 0.0, 24, deferred=True)


@pytest.mark.parametrize("fmt", ["int8", "int4"])
def test_quantised_layout_closed_form(fmt):
    """Single non-zero code per matrix: exposes byte/nibble order, scale indexing and the packer's transpose."""
    import torch

    d, I = 2048, 256
    cfg = CONFIGS["c4_dsv2lite_int4"].with_(n_layers=1, hidden=d, inter=I, shared_inter=0, n_experts=2, capacity=2,
                                            top_k=1, weight_fmt=fmt)
    store, dec = build(cfg)
    i, j1, j2, j3 = 133, 5, 1990, 1029
    if fmt == "int8":
        gq = torch.zeros(I, d, dtype=torch.int8); uq = torch.zeros(I, d, dtype=torch.int8)
        dq = torch.zeros(d, I, dtype=torch.int8)
        gq[i, j1], uq[i, j2], dq[j3, i] = 100, -50, 77
        gs = torch.ones(I, dtype=torch.float16); us = torch.ones(I, dtype=torch.float16)
        ds = torch.ones(d, dtype=torch.float16)
        gs[i], us[i], ds[j3] = 0.25, 0.5, 0.125
        wg, wu, wd = 100 * 0.25, -50 * 0.5, 77 * 0.125
    else:
        def codes(rows, cols):
            return torch.full((rows, cols // 2), 0x88, dtype=torch.uint8)  # all q = 0

        gq, uq, dq = codes(I, d), codes(I, d), codes(d, I)
        def put(m, r, c, q):
            b = int(m[r, c // 2])
            m[r, c // 2] = (b & 0xF0) | (q + 8) if c % 2 == 0 else (b & 0x0F) | ((q + 8) << 4)
        put(gq, i, j1, 7); put(uq, i, j2, -8); put(dq, j3, i, 5)
        gs = torch.ones(I, d // 128, dtype=torch.float16); us = torch.ones(I, d // 128, dtype=torch.float16)
        ds = torch.ones(d, I // 128, dtype=torch.float16)
        gs[i, j1 // 128], us[i, j2 // 128], ds[j3, i // 128] = 0.25, 0.5, 0.125
        wg, wu, wd = 7 * 0.25, -8 * 0.5, 5 * 0.125
    store.put_expert(0, 1, {"gate": (gq, gs), "up": (uq, us), "down": (dq, ds)})
    x = torch.zeros(d); x[j1], x[j2] = 0.75, 2.0
    xd, yd = x.to(torch.bfloat16).to(DEV), torch.zeros(d, dtype=torch.bfloat16, device=DEV)
    z = torch.tensor([0.0, 5.0], device=DEV)
    torch.cuda.synchronize()
    out = dec.route_step(0, logits=z)
    assert list(out.sel_expert[:1]) == [1]
    dec.expert_forward(0, xd, yd)
    dec.compute_stream.synchronize()
    a = wg * 0.75
    w = math.exp(5.0) / (1.0 + math.exp(5.0))
    expect = wd * (a / (1 + math.exp(-a))) * (wu * 2.0) * w
    y = yd.float().cpu().numpy()
    assert abs(y[j3] - expect) <= 5e-3 * abs(expect), (y[j3], expect)
    y[j3] = 0
    assert np.abs(y).max() <= 1e-3 * abs(expect), np.abs(y).max()
    dec.close()


def test_generators_are_device_independent():
    """The oracle regenerates weights on the CPU; the store is filled from the device: same bits."""
    import torch
    from synth import workloads

    for fmt in ("fp32", "bf16", "int8", "int4"):
        cfg = CONFIGS["c4_dsv2lite_int4"].with_(hidden=2048, inter=256, weight_fmt=fmt, seed=31)
        a, b = workloads.expert_weights(cfg, 1, 3, "cpu"), workloads.expert_weights(cfg, 1, 3, DEV)
        for k in ("gate", "up", "down"):
            ta = a[k] if isinstance(a[k], tuple) else (a[k],)
            tb = b[k] if isinstance(b[k], tuple) else (b[k],)
            for u, v in zip(ta, tb):
                assert torch.equal(u, v.cpu()), (fmt, k)
    cfg = CONFIGS["c2_qwen_bf16"].with_(n_layers=2)
    assert torch.equal(workloads.ar1_stream(cfg, 16), workloads.ar1_stream(cfg, 16, device=DEV).cpu())
    assert torch.equal(workloads.gate_weight(cfg, 1), workloads.gate_weight(cfg, 1, DEV).cpu())
