"""moe_expert_forward_static (the entry point for callers that cannot allocate) against moe_expert_forward, through
the C ABI: same kernels, same launch shape, same summation order, so the outputs must agree to the output
tolerance (1e-2 bf16 / 1e-5 fp32 relative to the largest element) - and in fact bit for bit.  Two calls in a row
share the library's fixed scratch array, the second with a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import experts as oexp
from synth import workloads
from synth.workloads import CONFIGS

from _gpu_common import DEV, OracleWeights, build

pytestmark = pytest.mark.gpu


def one_case(cfg, seed_tokens=2):
    import paper_2412_00099_amd as pkg

    print(f"case static entry {cfg.name} d={cfg.hidden} I={cfg.inter} shared={cfg.shared_inter} K={cfg.top_k}", flush=True)
    store, dec = build(cfg, lam=0.5)
    K = cfg.top_k
    xs = workloads.ar1_stream(cfg, seed_tokens)[:, 0].to(cfg.act_dtype).to(DEV)
    y_ctx = torch.zeros(cfg.hidden, dtype=cfg.act_dtype, device=DEV)
    y_static = torch.full((cfg.hidden,), 7.0, dtype=cfg.act_dtype, device=DEV)
    torch.cuda.synchronize()
    x = xs[-1]
    # the same token twice: the second time every selected expert is in its slot, so the context path is one launch
    for rep in range(2):
        out = dec.route_step(0, x=x)
        dec.expert_forward(0, x, y_ctx)
    dec.compute_stream.synchronize()
    assert out.n_miss == 0
    slots, weights = list(out.sel_slot[:K]), list(out.sel_weight[:K])
    stream = C.c_void_p(dec.compute_stream.cuda_stream)
    pkg.moe_expert_forward_static(store.wfmt, store.afmt, cfg.hidden, cfg.inter, cfg.shared_inter, K,
                                  C.c_void_p(store.pools[0].data_ptr()), cfg.capacity,
                                  C.c_void_p(store.shared[0].data_ptr()) if cfg.shared_inter else None,
                                  slots, weights, C.c_void_p(x.data_ptr()), C.c_void_p(y_static.data_ptr()), stream)
    dec.compute_stream.synchronize()
    a, b = y_ctx.float().cpu().numpy(), y_static.float().cpu().numpy()
    tol = 1e-5 if cfg.act_fmt == "fp32" else 1e-2
    assert oexp.rel_err(b, a) <= tol
    assert np.array_equal(a, b), "same kernels in the same order: expected identical bits"
    # and against the oracle, so that a mistake shared by both entry points does not pass
    ow = OracleWeights(cfg)
    experts = [ow.expert(0, int(e)) for e in out.sel_expert[:K]]
    y_ref = oexp.moe_output(x.float().cpu().numpy(), experts, np.array(weights, np.float64), ow.shared(0))
    assert oexp.rel_err(b, y_ref) <= tol
    # argument errors: nothing is launched
    bad = list(slots)
    bad[0] = cfg.capacity
    with pytest.raises(pkg.MoEError) as e:
        pkg.moe_expert_forward_static(store.wfmt, store.afmt, cfg.hidden, cfg.inter, cfg.shared_inter, K,
                                      C.c_void_p(store.pools[0].data_ptr()), cfg.capacity, None if not cfg.shared_inter
                                      else C.c_void_p(store.shared[0].data_ptr()), bad, weights,
                                      C.c_void_p(x.data_ptr()), C.c_void_p(y_static.data_ptr()), stream)
    assert e.value.code == pkg.MOE_EINVAL
    dec.close()


def test_static_entry_two_calls_second_smaller():
    big = CONFIGS["c2_qwen_bf16"].with_(n_layers=1, hidden=2048, n_experts=12, inter=160, shared_inter=320, capacity=6,
                                        top_k=4, seed=8101)
    one_case(big)
    small = CONFIGS["c1_single_fp32"].with_(n_layers=1, hidden=256, n_experts=8, inter=40, shared_inter=0, capacity=4,
                                            top_k=2, seed=8102)
    one_case(small)
    # a third call with the larger shape again: the scratch array keeps the smaller call's rows, which must not leak in
    one_case(big.with_(weight_fmt="int8", inter=96, shared_inter=96, seed=8103))


def test_static_entry_refuses_sizes_beyond_its_scratch():
    import paper_2412_00099_amd as pkg

    x = torch.zeros(8192, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(pkg.MoEError) as e:
        pkg.moe_expert_forward_static(pkg.MOE_W_BF16, pkg.MOE_A_BF16, 8192, 64, 0, 1, C.c_void_p(x.data_ptr()), 1, None,
                                      [0], [1.0], C.c_void_p(x.data_ptr()), C.c_void_p(x.data_ptr()), None)
    assert e.value.code == pkg.MOE_EINVAL and "scratch" in str(e.value)
