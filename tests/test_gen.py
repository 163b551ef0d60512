"""The seeded input generators: determinism, shapes and the structure the workloads ask for."""
import numpy as np
import torch

from gen import rng, workloads
from gen.graphs import power_law_degrees, power_law_relation, reverse_relation


def test_streams_are_stateless_and_named():
    a = rng.normal_table(1000, 8, "w", "x")
    b = rng.normal_table(1000, 8, "w", "x")
    c = rng.normal_table(1000, 8, "w", "y")
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    # block-wise fill: a longer table starts with the same rows
    big = rng.normal_table((1 << 16) + 10, 8, "w", "x")
    assert np.array_equal(big[:1000], a)


def test_bf16_rounding_matches_library_conversion():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]   # ties: to even
    ours = rng.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours.view(np.uint32), ref.view(np.uint32))
    bits = rng.f32_to_bf16_bits(x)
    assert np.array_equal(rng.bf16_bits_to_f32(bits), ours)


def test_power_law_degrees_sum_and_tail():
    g = rng.stream("t", "deg")
    deg = power_law_degrees(200_000, 1_000_000, 2.1, g)
    assert deg.sum() == 1_000_000 and deg.min() >= 0
    assert (deg <= 2).mean() > 0.4          # most rows are tiny
    assert deg.max() > 5_000                # and a few are hubs
    # log-log slope of the degree histogram between 4 and 256 is about -2.1
    ks = np.array([4, 8, 16, 32, 64, 128])
    cnt = np.array([((deg >= k) & (deg < 2 * k)).sum() for k in ks], dtype=np.float64)
    slope = np.polyfit(np.log(ks), np.log(cnt / ks), 1)[0]
    assert -2.6 < slope < -1.6, slope


def test_reverse_relation_is_exact_transpose():
    r = power_law_relation("r", 0, 1, 300, 200, 2000, 2.0, "t")
    rv = reverse_relation("rv", r, 300)
    s, d = r.edge_list()
    s2, d2 = rv.edge_list()
    a = np.stack([s, d], 1)
    b = np.stack([d2, s2], 1)
    assert np.array_equal(a[np.lexsort((a[:, 1], a[:, 0]))], b[np.lexsort((b[:, 1], b[:, 0]))])
    assert rv.src_type == 1 and rv.dst_type == 0 and rv.rowptr.shape[0] == 301


def test_config_shapes():
    p = workloads.config1()
    assert [t.num_nodes for t in p.graph.ntypes] == [2000, 1000, 500]
    assert all(r.num_edges == 5000 for r in p.graph.relations)
    assert p.edge_features() == 4 * 5000 * 32
    p3 = workloads.config3("bf16", scale=0.01)
    assert len(p3.graph.relations) == 7 and p3.op == "mean" and p3.d_out == 256
    assert np.array_equal(p3.tables[0], rng.round_to_bf16(p3.tables[0]))
    p4 = workloads.config4(scale=0.002)
    assert len(p4.graph.relations) == 12 and len(p4.graph.ntypes) == 7 and p4.op == "sum"
    assert sorted(w.shape[0] for w in p4.W) == sorted([7, 24, 64, 64, 512, 789] + [300] * 6)
