"""The seeded input generators: determinism, shape of the distributions,
validity of sampled blocks."""
import numpy as np

from bifeat_inputs import (FeatureSpec, feature_chunk, feature_rows, column_params,
                           PowerLawGraph, UniformGraph, sample_blocks, draw_seeds,
                           WORKLOADS, make_graph)


def test_rows_are_a_pure_function_of_their_index():
    spec = FeatureSpec(10_000, 100, 0)
    a = feature_chunk(spec, 0, 300)
    b = feature_rows(spec, np.array([299, 0, 17, 17]))
    assert np.array_equal(b, a[[299, 0, 17, 17]])
    big = feature_rows(FeatureSpec(244_000_000, 768, 0, "f16"), np.array([243_999_999, 5]))
    assert big.dtype == np.float16 and big.shape == (2, 768) and np.isfinite(big).all()
    assert not np.array_equal(a, feature_chunk(FeatureSpec(10_000, 100, 1), 0, 300))


def test_columns_look_gaussian_with_their_own_location_and_scale():
    spec = FeatureSpec(20_000, 32, 0)
    x = feature_chunk(spec, 0, 20_000).astype(np.float64)
    mu, sigma = column_params(0, 32)
    assert np.all((mu >= -1) & (mu < 1) & (sigma >= 0.5) & (sigma < 2))
    z = (x - mu) / sigma
    assert np.allclose(z.mean(0), 0, atol=0.03) and np.allclose(z.std(0), 1, atol=0.03)
    assert np.abs(z).max() < 3.47
    assert abs((np.abs(z) < 1).mean() - 0.683) < 0.02


def test_fp16_table_is_rounded_fp32_table():
    a = feature_chunk(FeatureSpec(1000, 64, 0, "f32"), 10, 50)
    b = feature_chunk(FeatureSpec(1000, 64, 0, "f16"), 10, 50)
    assert np.array_equal(a.astype(np.float16), b)


def test_power_law_graph_degrees_and_endpoints():
    g = PowerLawGraph(2_400_000, 15, 2.1, 10_000, 0)
    u = np.arange(0, g.N, 7)
    d = g.degree(u)
    assert abs(d.mean() - 15) < 0.3 and d.min() >= 1 and d.max() == 10_000
    # tail exponent: P(deg >= x) ~ x^-(alpha-1)
    p1, p2 = (d >= 20).mean(), (d >= 200).mean()
    assert abs(np.log10(p1 / p2) - 1.1) < 0.1
    # endpoints are drawn in proportion to degree: mean degree of an endpoint
    # is E[d^2]/E[d], far above the node average
    nb = g.neighbor(u[:200_000], np.zeros(200_000, np.int64))
    assert nb.min() >= 0 and nb.max() < g.N
    dn = g.degree(nb).astype(np.float64)
    want = (d.astype(np.float64) ** 2).mean() / d.mean()
    assert abs(dn.mean() / want - 1) < 0.15
    # the rank <-> id scattering is a bijection
    r = np.arange(0, 100_000)
    assert np.array_equal(g._rank(g._node(r)).astype(np.int64), r)


def test_sampled_blocks_are_valid():
    for name in ["tiny", "mid"]:
        w = WORKLOADS[name]
        g = make_graph(w)
        seeds = draw_seeds(g, w.batch, w.seed, 3, w.seed_mode)
        assert len(np.unique(seeds)) == w.batch
        blocks, inputs = sample_blocks(g, seeds, w.fanouts, w.seed, 3)
        assert np.array_equal(blocks[0].dst, np.unique(seeds))
        frontier = blocks[0].dst
        for b, f in zip(blocks, w.fanouts):
            assert np.array_equal(b.dst, frontier)
            n = np.diff(b.indptr)
            assert np.array_equal(n, np.minimum(g.degree(b.dst), f))
            assert b.indices.min() >= 0 and b.indices.max() < w.N
            frontier = np.unique(np.concatenate([b.dst, b.indices]))
        assert np.array_equal(inputs, frontier)
        again, _ = sample_blocks(g, seeds, w.fanouts, w.seed, 3)
        assert np.array_equal(again[-1].indices, blocks[-1].indices)
        other, _ = sample_blocks(g, seeds, w.fanouts, w.seed, 4)
        assert name == "tiny" or not np.array_equal(other[-1].indices, blocks[-1].indices)


def test_uniform_graph_slots_without_replacement():
    g = UniformGraph(10_000, 15, 0)
    seeds = draw_seeds(g, 64, 0, 0)
    (b,), _ = sample_blocks(g, seeds, (10,), 0, 0)
    assert np.all(np.diff(b.indptr) == 10)
    # the 10 sampled neighbours of a node are among its 15, from distinct slots
    for v in range(5):
        full = g.neighbor(np.full(15, b.dst[v]), np.arange(15))
        got = b.indices[b.indptr[v]:b.indptr[v + 1]]
        pos = [int(np.nonzero(full == x)[0][0]) for x in got]
        assert all(x in full for x in got) and pos == sorted(pos)


def test_full_csr_lists_every_slot_after_the_node_itself():
    from bifeat_inputs import full_csr
    g = PowerLawGraph(500, 6.0, seed=4)
    indptr, indices = full_csr(g, chunk=128)
    u = np.arange(500, dtype=np.int64)
    assert np.array_equal(np.diff(indptr), g.degree(u) + 1)
    assert np.array_equal(indices[indptr[:-1]], u)
    for v in (0, 127, 128, 499):
        d = int(g.degree(np.array([v]))[0])
        want = g.neighbor(np.full(d, v, np.int64), np.arange(d, dtype=np.int64))
        assert np.array_equal(indices[indptr[v] + 1:indptr[v + 1]], want)
    ip2, ix2 = full_csr(g, self_loops=False)
    assert np.array_equal(np.diff(ip2), g.degree(u))
    assert np.array_equal(ix2[ip2[7]:ip2[8]], indices[indptr[7] + 1:indptr[8]])
