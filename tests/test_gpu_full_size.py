"""Full per-layer shapes of the workloads, in the launch configuration bench.py times: routing checked on every
token, outputs on sampled (token, layer) pairs the oracle can afford.  Layers are independent in these runs
(each fed its own exogenous AR(1) stream), so one or two layers exercise every kernel at its real shape: the
benchmarked Qwen1.5-MoE shape in bf16, and the OLMoE (bf16, top-8, no shared expert), DeepSeek-V2-Lite (int4,
group 128, two shared experts) and Mixtral (int8, d = 4096, 176 MB experts) shapes."""
import os

import pytest

from synth.workloads import CONFIGS

from test_gpu_route import free_run
from test_gpu_stack import run_in_launch_boundary

pytestmark = pytest.mark.gpu


def test_c2_full_layer_shape():
    cfg = CONFIGS["c2_qwen_bf16"].with_(n_layers=2)
    print("case c2 full per-layer shape, 2 layers, 40 tokens", flush=True)
    free_run(cfg, 0.5, 40, top_j=0, check_outputs_every=13, deferred=True)  # as bench.py drives it


def test_c2_full_layer_shape_coupled_stack():
    """The launch configuration bench.py times: residual stream carried from layer to layer, the layer boundary in
    the first workgroup of the expert launch (chosen by the library's own rule for this shape), misses filled on the
    side stream.  Routing, h, x and logits checked on every layer-token, outputs on every 5th."""
    if os.environ.get("MOE_FUSE_BOUNDARY") == "0":
        pytest.skip("the in-launch boundary is switched off in the environment")
    cfg = CONFIGS["c2_qwen_bf16"].with_(n_layers=2)
    print("case c2 full per-layer shape, coupled stack, 2 layers, 10 tokens", flush=True)
    ties, misses = run_in_launch_boundary(cfg, 10, 0.5, outputs_every=5, force=False)
    assert misses >= cfg.top_k * cfg.n_layers


@pytest.mark.parametrize("capacity", [16, 32, 48])
def test_c3_full_layer_shape(capacity):
    """The three cache sizes of the workload (cache-size ablation, Sec. 4.8) at the full layer shape."""
    cfg = CONFIGS["c3_olmoe_bf16"].with_(n_layers=1, capacity=capacity)
    print(f"case c3 full per-layer shape, cache {capacity}, 1 layer, 24 tokens", flush=True)
    free_run(cfg, 0.5, 24, top_j=0, check_outputs_every=11, deferred=True)


def test_c4_full_layer_shape():
    cfg = CONFIGS["c4_dsv2lite_int4"].with_(n_layers=1)
    print("case c4 full per-layer shape, 1 layer, 24 tokens", flush=True)
    free_run(cfg, 0.5, 24, top_j=0, check_outputs_every=11, deferred=True)


def test_c5_full_layer_shape():
    cfg = CONFIGS["c5_mixtral_int8"].with_(n_layers=1)
    print("case c5 full per-layer shape, 1 layer, 6 tokens (outputs: first and last)", flush=True)
    free_run(cfg, 0.5, 6, top_j=0, check_outputs_every=5, deferred=True)
