"""Pins for the expert/MoE-output oracle: library routines, closed forms, explicit loops."""
import math

import numpy as np
import pytest
import torch

from oracle import experts, rerank, stack


def test_swiglu_against_torch_double():
    g = torch.Generator().manual_seed(1)
    d, I = 24, 40  # non-square: a transposed operand cannot even be multiplied
    x = torch.randn(d, generator=g, dtype=torch.float64)
    wg = torch.randn(I, d, generator=g, dtype=torch.float64)
    wu = torch.randn(I, d, generator=g, dtype=torch.float64)
    wd = torch.randn(d, I, generator=g, dtype=torch.float64)
    ref = wd @ (torch.nn.functional.silu(wg @ x) * (wu @ x))
    got = experts.swiglu_expert(x.numpy(), wg.numpy(), wu.numpy(), wd.numpy())
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_swiglu_explicit_loops_tiny():
    r = np.random.default_rng(3)
    d, I = 3, 5
    x, wg, wu, wd = r.standard_normal(d), r.standard_normal((I, d)), r.standard_normal((I, d)), r.standard_normal((d, I))
    y = [0.0] * d
    for i in range(I):
        a = sum(wg[i][j] * x[j] for j in range(d))
        b = sum(wu[i][j] * x[j] for j in range(d))
        h = a / (1.0 + math.exp(-a)) * b
        for j in range(d):
            y[j] += wd[j][i] * h
    np.testing.assert_allclose(experts.swiglu_expert(x, wg, wu, wd), y, rtol=1e-12)


def test_closed_forms():
    d, I = 4, 6
    x = np.array([1.0, -2.0, 0.5, 3.0])
    # zero gate -> silu(0) = 0 -> zero output whatever up/down are
    assert np.all(experts.swiglu_expert(x, np.zeros((I, d)), np.ones((I, d)), np.ones((d, I))) == 0)
    # gate row picks x[3]=3, up row picks x[1]=-2, down routes unit i=2 to output 0 with gain 5
    wg = np.zeros((I, d)); wu = np.zeros((I, d)); wd = np.zeros((d, I))
    wg[2, 3] = 1; wu[2, 1] = 1; wd[0, 2] = 5
    y = experts.swiglu_expert(x, wg, wu, wd)
    assert np.allclose(y, [5 * (3 / (1 + math.exp(-3))) * -2, 0, 0, 0])


def test_moe_output_weights_and_shared():
    r = np.random.default_rng(4)
    d, I = 8, 12
    x = r.standard_normal(d)
    es = [{k: r.standard_normal((I, d) if k != "down" else (d, I)) for k in ("gate", "up", "down")} for _ in range(3)]
    sh = {k: r.standard_normal((2 * I, d) if k != "down" else (d, 2 * I)) for k in ("gate", "up", "down")}
    w = [0.5, 0.25, 0.125]
    parts = [experts.swiglu_expert(x, e["gate"], e["up"], e["down"]) for e in es]
    ref = 0.5 * parts[0] + 0.25 * parts[1] + 0.125 * parts[2] + experts.swiglu_expert(x, sh["gate"], sh["up"], sh["down"])
    np.testing.assert_allclose(experts.moe_output(x, es, w, sh), ref, rtol=1e-12)


def test_dequantize_int8_rows():
    q = np.array([[1, -2, 127], [-127, 0, 5]], np.int8)
    s = np.array([0.5, 2.0], np.float16)
    np.testing.assert_array_equal(experts.dequantize((q, s)), [[0.5, -1.0, 63.5], [-254.0, 0.0, 10.0]])


def test_dequantize_int4_nibble_order_and_groups():
    cols = 256
    packed = np.full((1, cols // 2), 0x88, np.uint8)  # all q = 0
    packed[0, 0] = 0x2F  # column 0: low nibble 15 -> q=+7 ; column 1: high nibble 2 -> q=-6
    packed[0, 64] = 0x80 | 0x9  # column 128 (second group): low nibble 9 -> q=+1
    s = np.array([[0.5, 4.0]], np.float16)
    w = experts.dequantize((packed, s))
    assert w.shape == (1, cols)
    assert w[0, 0] == 3.5 and w[0, 1] == -3.0 and w[0, 128] == 4.0
    assert np.count_nonzero(w) == 3


def test_quantizers_round_trip_within_half_step():
    from synth import workloads

    g = torch.Generator().manual_seed(0)
    w = torch.randn(16, 256, generator=g) * 0.02
    q, s = workloads.quantize_int8(w)
    deq = experts.dequantize((q.numpy(), s.numpy()))
    assert np.abs(deq - w.numpy()).max() <= 0.5 * float(s.float().max()) * 1.001
    p, s4 = workloads.quantize_int4(w)
    deq4 = experts.dequantize((p.numpy(), s4.numpy()))
    # symmetric range [-8, 7]: the positive maximum clips by up to one step
    assert np.abs(deq4 - w.numpy()).max() <= float(s4.float().max()) * 1.001


def test_promote_and_maxrank_golden():
    vals = {}
    for line in open(__file__.rsplit("/", 1)[0] + "/golden/maxrank_example.txt"):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":")
        vals[k.strip()] = [int(t) for t in v.split()]
    r, cache = vals["ranking"], set(vals["cache"])
    M, K, J = vals["M"][0], vals["K"][0], vals["J"][0]
    step1 = rerank.promote([e for e in r[:M] if e in cache], r)
    assert step1 == vals["after_cache_promote"]
    assert rerank.promote(r[:J], step1) == vals["after_topj_promote"]
    out = rerank.max_rank(r, cache, M, J)
    assert out == vals["after_topj_promote"] and out[:K] == vals["selected"]


def test_cumsum_rank():
    w = [0.5, 0.3, 0.1, 0.1]
    assert rerank.cumsum_rank(w, 0.5) == 1
    assert rerank.cumsum_rank(w, 0.79) == 2
    assert rerank.cumsum_rank(w, 0.85) == 3
    assert rerank.cumsum_rank(w, 2.0) == 4
    # flat distribution -> larger M than a peaked one (App. B)
    assert rerank.cumsum_rank([0.25] * 4, 0.7) > rerank.cumsum_rank([0.9, 0.05, 0.03, 0.02], 0.7)
    r = rerank.cumsum_threshold([0, 1, 2, 3], dict(enumerate(w)), {2, 3}, 0.85, 1)
    assert r == [0, 2, 1, 3]


def test_prune_structure():
    """Pruning baseline (Sec. 4.2): no value is printed in the paper (parity unpinned); what the definition itself
    fixes is pinned here - a prefix of the ranking, ranks counted from 1 so that h = 2 keeps one expert and h = K
    still drops the last, h = K + 1 is the original routing, and the miss rate is normalised by K."""
    r = [4, 2, 7, 1, 0]
    K = 3
    assert rerank.prune(r, K, 2) == [4]
    assert rerank.prune(r, K, 3) == [4, 2]
    assert rerank.prune(r, K, K + 1) == r[:K] == rerank.prune(r, K, 9)
    for h in range(2, K + 2):
        kept = rerank.prune(r, K, h)
        assert kept == r[: len(kept)] and len(kept) == min(K, h - 1)
    with pytest.raises(AssertionError):
        rerank.prune(r, K, 1)
    assert rerank.pruned_miss_rate(6, 4, 3) == 0.5  # 6 misses over 4 tokens of K = 3, whatever was kept


def test_pruned_miss_rate_bounds():
    """A pruned token touches at most h - 1 experts, so its miss rate normalised by K is at most (h - 1) / K; with
    h = K + 1 the pruned run is the original routing, miss for miss."""
    from oracle import eviction

    rng = np.random.default_rng(11)
    N, K, C, T = 12, 4, 6, 300
    z = np.cumsum(rng.normal(size=(T, N)), axis=0) * 0.3 + rng.normal(size=(T, N))
    ranks = [np.argsort(-row, kind="stable").tolist() for row in z]
    full, _ = eviction.lru_list_misses([r[:K] for r in ranks], C)
    for h in range(2, K + 2):
        m, _ = eviction.lru_list_misses([rerank.prune(r, K, h) for r in ranks], C)
        assert rerank.pruned_miss_rate(m, T, K) <= (h - 1) / K
        if h == K + 1:
            assert m == full


def test_stack_glue():
    h = np.array([3.0, 4.0])
    x = stack.rmsnorm(h)
    assert abs(np.mean(x * x) - 1.0) < 1e-6
    np.testing.assert_allclose(stack.next_hidden([1, 2], [0.5, 0.5], [2, -2]), [2.5, 1.5])
