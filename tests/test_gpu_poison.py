"""Use-before-fill guard: with MOE_POISON_FILLS=1 the library overwrites a slot with NaN patterns right before the
copy that fills it.  A kernel that computed from a slot before its fill had landed would then put NaNs into y, which
the output comparisons of these runs (misses on most tokens: small caches) cannot pass.  Pass 0 of a layer does read
the records of experts that are still being filled - by design, without using them - so this also checks that those
values go nowhere."""
import pytest

from synth.workloads import CONFIGS

from test_gpu_prompt import run_prompt_outputs
from test_gpu_stack import run_in_launch_boundary

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,hidden,inter", [("c2_qwen_bf16", 2048, 96), ("c4_dsv2lite_int4", 2048, 128),
                                               ("c5_mixtral_int8", 1024, 64)])
def test_decode_with_poisoned_fills(name, hidden, inter, monkeypatch):
    monkeypatch.setenv("MOE_POISON_FILLS", "1")
    base = CONFIGS[name]
    cfg = base.with_(n_layers=2, hidden=hidden, n_experts=12, inter=inter,
                     shared_inter=2 * inter if base.shared_inter else 0, capacity=5, top_k=min(base.top_k, 4),
                     seed=7700 + hidden + inter)
    ties, misses = run_in_launch_boundary(cfg, 12, 0.0, monkeypatch=monkeypatch)
    assert misses > cfg.top_k * cfg.n_layers  # LRU routing on a cache of five: refills well beyond the cold ones


def test_prompt_phase_with_poisoned_fills(monkeypatch):
    monkeypatch.setenv("MOE_POISON_FILLS", "1")
    cfg = CONFIGS["c2_qwen_bf16"].with_(n_layers=1, hidden=1024, n_experts=10, inter=48, shared_inter=96, top_k=2,
                                        capacity=3, seed=7801)
    run_prompt_outputs(cfg, 0.0, [8, 37, 128, 16])
