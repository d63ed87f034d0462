"""The seeded input generators: reproducible, right shapes and statistics."""
import numpy as np
import torch

from synth import rng, workloads
from synth.workloads import CONFIGS


def test_splitmix_reference_values():
    # splitmix64 with seed 0: the first outputs of the published generator
    state, outs = 0, []
    for _ in range(3):
        state = (state + 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
        outs.append(rng._mix64_int(state))
    assert outs[0] == 0xE220A8397B1DCDAF and outs[1] == 0x6E789E6AA1B965F4
    t = rng.mix64(torch.tensor([rng._s64(0x9E3779B97F4A7C15)], dtype=torch.int64))
    assert (int(t[0]) & ((1 << 64) - 1)) == outs[0]


def test_normal_statistics_and_determinism():
    a = rng.standard_normal(rng.stream_key(1, 2), 200_000)
    b = rng.standard_normal(rng.stream_key(1, 2), 200_000)
    c = rng.standard_normal(rng.stream_key(1, 3), 200_000)
    assert torch.equal(a, b) and not torch.equal(a, c)
    assert abs(float(a.mean())) < 0.01 and abs(float(a.std()) - 1.0) < 0.01
    assert abs(float((a.abs() > 1.96).float().mean()) - 0.05) < 0.004
    # offset addressing: a slice of the stream equals the stream generated at that offset
    assert torch.equal(a[1000:1100], rng.standard_normal(rng.stream_key(1, 2), 100, offset=1000))


def test_weight_shapes_and_formats():
    cfg = CONFIGS["c1_single_fp32"]
    e = workloads.expert_weights(cfg, 0, 3)
    assert e["gate"].shape == (512, 256) and e["down"].shape == (256, 512) and e["gate"].dtype == torch.float32
    assert abs(float(e["gate"].std()) - 0.02) < 0.001
    small = CONFIGS["c4_dsv2lite_int4"].with_(hidden=256, inter=128, shared_inter=256)
    q, s = workloads.expert_weights(small, 0, 0)["down"]
    assert q.shape == (256, 64) and q.dtype == torch.uint8 and s.shape == (256, 1) and s.dtype == torch.float16
    q8, s8 = workloads.expert_weights(small.with_(weight_fmt="int8"), 0, 0)["gate"]
    assert q8.shape == (128, 256) and q8.dtype == torch.int8 and s8.shape == (128,)
    sh = workloads.shared_weights(small.with_(weight_fmt="bf16"), 1)
    assert sh["up"].shape == (256, 256) and sh["up"].dtype == torch.bfloat16
    assert workloads.gate_weight(small, 0).shape == (64, 256)


def test_ar1_is_stationary_with_the_asked_correlation():
    cfg = CONFIGS["c1_single_fp32"]
    a = workloads.ar1_stream(cfg, 256).numpy()[:, 0, :]
    assert a.shape == (256, 256)
    assert abs(a.std() - 1.0) < 0.03
    corr = np.mean(a[1:] * a[:-1]) / np.mean(a * a)
    assert abs(corr - 0.9) < 0.02


def test_configs_match_the_paper_table_shapes():
    c2, c5 = CONFIGS["c2_qwen_bf16"], CONFIGS["c5_mixtral_int8"]
    assert 3 * c2.hidden * c2.inter == 8_650_752  # 8.6 M parameters per expert (Table 1)
    assert 3 * c5.hidden * c5.inter == 176_160_768  # 176 M (Table 1)
    assert c2.capacity * 2 == c2.n_experts and c5.capacity * 2 == c5.n_experts
    assert len(workloads.initial_residents(c2, 0, 30)) == 30
