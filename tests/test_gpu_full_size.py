"""Full per-layer shape of the benchmarked workload (Qwen1.5-MoE-shaped, bf16), in the launch configuration
bench.py times: routing checked on every token, outputs on sampled (token, layer) pairs the oracle can
afford.  Layers are independent in this run (each fed its own exogenous AR(1) stream), so two layers of
the 24 exercise every kernel at its real shape."""
import pytest

from synth.workloads import CONFIGS

from test_gpu_route import free_run

pytestmark = pytest.mark.gpu


def test_c2_full_layer_shape():
    cfg = CONFIGS["c2_qwen_bf16"].with_(n_layers=2)
    print("case c2 full per-layer shape, 2 layers, 40 tokens", flush=True)
    free_run(cfg, 0.5, 40, top_j=0, check_outputs_every=13, deferred=True)  # as bench.py drives it
