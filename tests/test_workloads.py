"""The synthetic input generator: deterministic, right shapes, right coarse statistics."""
import numpy as np

import workloads


def test_tiny_is_deterministic_and_shaped():
    cfg = workloads.CONFIGS["tiny"]
    a = workloads.make_all(cfg, seed=0)
    b = workloads.make_all(cfg, seed=0)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    E, perms, topfreq, H = a
    assert E.shape == (1000, 64) and E.dtype == np.float32
    assert perms.shape == (16, 8) and perms.dtype == np.int32
    assert all(len(set(r.tolist())) == 8 and r.min() >= 0 and r.max() < 64 for r in perms)
    assert topfreq.tolist() == list(range(50))
    assert H.shape == (20, 4, 64) and H.dtype == np.float32
    assert not np.array_equal(E, workloads.make_embeddings(cfg, seed=1))


def test_cluster_structure_and_scales():
    cfg = workloads.CONFIGS["tiny"]
    E = workloads.make_embeddings(cfg, 0)
    same = np.std(E[0] - E[32])        # same centre: two noise draws
    diff = np.std(E[0] - E[1])
    assert 0.3 < same < 0.55 and diff > 1.0


def test_zipf_targets_are_head_heavy():
    cfg = workloads.CONFIGS["paper"]
    w = workloads.zipf_targets(cfg, 20000, np.random.default_rng(0))
    assert w.min() >= 0 and w.max() < cfg.V
    assert (w == 0).mean() > 0.08 and (w < 1000).mean() > 0.5


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.14159], dtype=np.float32)
    bits = workloads.f32_to_bf16_bits(x)
    back = workloads.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: goes to even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert back[:4].tolist() == [1.0, 1.0, 1.015625, -2.5]
    assert abs(back[4] - 3.14159) < 2 ** -7 * 2


def test_config_table_matches_the_benchmark_definitions():
    c = workloads.CONFIGS
    assert (c["paper"].d, c["paper"].V, c["paper"].B, c["paper"].S) == (1000, 40000, 12, 1)
    assert (c["paper"].K, c["paper"].P, c["paper"].W, c["paper"].T) == (8, 32, 8, 1000)
    assert (c["batched"].S, c["batched"].B) == (32, 10)
    assert (c["widebeam"].V, c["widebeam"].B, c["widebeam"].S, c["widebeam"].K) == (100000, 50, 4, 16)
    assert (c["largevocab"].d, c["largevocab"].V, c["largevocab"].R) == (1024, 200000, 640)
    assert c["largevocab"].e_dtype == workloads.BF16
    assert all(v.u == 4 and v.threshold == 1 for n, v in c.items() if n != "paperscale")
    ps = c["paperscale"]                      # the paper's {K, u, W} = {8, 3, 500} with a hit threshold
    assert (ps.d, ps.V, ps.B, ps.K, ps.u, ps.W, ps.threshold) == (1000, 40000, 12, 8, 3, 500, 5)
