"""GPU parity for the layers after the first and the aggregation scale profile
(Appendix A.1, A.3, A.5): fp32-row aggregation, two-hop chains that start from
the packed table, and the profiling run, each against the CPU oracle."""
import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import (FeatureSpec, PowerLawGraph, UniformGraph, draw_seeds, feature_chunk,
                           full_csr, sample_blocks)
from helpers import assert_close, gpu_build_table, oracle_uniform_table, random_csr, scheme_of

pytestmark = pytest.mark.gpu

REL_TOL = 1e-5


@pytest.fixture(scope="module")
def bf():
    import paper_2207_14696_amd as m
    m.load_library()
    return m


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


def _assert_rows_close(got, want, x, indptr, indices, as_sum, what):
    # |gpu - oracle| <= 1e-5 * max(|oracle|, mean over the list of |x|) (times the list
    # length for the sum): the scale the rounding of a sum is measured against
    ref = orc.aggregate_rows(np.abs(x), indptr, indices, sum=as_sum).astype(np.float64)
    bound = REL_TOL * np.maximum(np.abs(want.astype(np.float64)), ref)
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside 1e-5; worst {(err / np.maximum(bound, 1e-300)).max():.3g}"


@pytest.mark.parametrize("as_sum", [False, True])
@pytest.mark.parametrize("D", [128, 100, 37, 768, 600, 4, 1, 1028])
def test_aggregate_rows_matches_the_oracle(bf, torch, D, as_sum):
    rng = np.random.default_rng(D)
    N, V = 3000, 1501
    x = (rng.standard_normal((N, D)) * rng.uniform(0.1, 10, D)).astype(np.float32)
    indptr, indices = random_csr(V, N, 20, rng, hubs=(300, 4500))
    want = orc.aggregate_rows(x, indptr, indices, sum=as_sum)
    dx = torch.from_numpy(x).cuda()
    got = bf.aggregate_rows(dx, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(),
                            sum=as_sum).cpu().numpy()
    assert not got[0].any()
    _assert_rows_close(got, want, x, indptr, indices, as_sum, f"D={D}")


def test_aggregate_rows_edge_cases(bf, torch):
    x = torch.arange(40, dtype=torch.float32, device="cuda").reshape(10, 4)
    empty = torch.zeros(1, dtype=torch.int64, device="cuda")
    none = torch.zeros(0, dtype=torch.int64, device="cuda")
    assert bf.aggregate_rows(x, empty, none).shape == (0, 4)
    # every list empty: all-zero rows, written (the buffer starts out as ones)
    out = torch.ones((5, 4), dtype=torch.float32, device="cuda")
    bf.aggregate_rows(x, torch.zeros(6, dtype=torch.int64, device="cuda"), none, out=out)
    assert not out.cpu().numpy().any()
    # a single neighbour is that row, bit for bit; unaligned views take the scalar path
    idx = torch.tensor([7, 0, 9], dtype=torch.int64, device="cuda")
    ptr = torch.arange(4, dtype=torch.int64, device="cuda")
    assert torch.equal(bf.aggregate_rows(x, ptr, idx), x[idx])
    flat = torch.arange(41, dtype=torch.float32, device="cuda")
    shifted = flat[1:].reshape(10, 4)                          # 4-byte aligned only
    assert torch.equal(bf.aggregate_rows(shifted, ptr, idx), shifted[idx])


@pytest.mark.parametrize("kind,bits,D", [("uniform", 4, 128), ("uniform", 2, 100), ("log", 1, 64)])
def test_two_hop_chain_from_the_packed_table(bf, torch, kind, bits, D):
    # layer 1 aggregates decoded rows of the packed table over the outer block; layer 2
    # aggregates layer 1's output over the seed block, its lists renumbered to rows of
    # that output (the frontier is sorted, so a binary search renumbers them)
    N = 20000
    spec = FeatureSpec(N, D, 3)
    x = feature_chunk(spec, 0, N)
    if kind == "uniform":
        _, _, s, codes = oracle_uniform_table(spec, bits)
        q = bf.Quantizer(scheme_of("uniform", bits), D)
    else:
        e_min, e_max = orc.log_range(orc.log_fit(x))
        T, Vt = orc.log_tables(e_min, e_max, bits)
        codes = orc.pack(orc.log_encode(x, bits, T), bits)
        s = orc.Scheme.log(D, Vt, bits)
        q = bf.Quantizer(scheme_of("log", bits), D)
    from bifeat_inputs.device import DeviceTable
    dcodes = gpu_build_table(q, DeviceTable(spec), N, 8192)
    assert np.array_equal(dcodes.cpu().numpy(), codes)
    g = PowerLawGraph(N, 12.0, seed=5)
    seeds = draw_seeds(g, 512, 5, 0)
    blocks, _ = sample_blocks(g, seeds, [10, 15], 5, 0)
    inner, outer = blocks[0], blocks[1]
    local = np.searchsorted(outer.dst, inner.indices)
    assert np.array_equal(outer.dst[local], inner.indices)
    h1_want = orc.gather_mean(s, codes, outer.indptr, outer.indices)
    h2_want = orc.aggregate_rows(h1_want, inner.indptr, local)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    h1 = q.gather_mean(dcodes, cu(outer.indptr), cu(outer.indices))
    h2 = bf.aggregate_rows(h1, cu(inner.indptr), cu(local))
    assert_close(h1.cpu().numpy(), h1_want, s, "layer 1")
    # layer 2 inherits layer 1's rounding once more
    A = np.abs(orc.gather_dequant(s, codes, np.arange(N))).max(axis=0).astype(np.float64)[None, :]
    err = np.abs(h2.cpu().numpy().astype(np.float64) - h2_want.astype(np.float64))
    assert (err <= 2 * REL_TOL * np.maximum(np.abs(h2_want), A)).all()


def _lists(rows):
    indptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int64)
    return indptr, np.array([j for r in rows for j in r], dtype=np.int64)


def test_scale_profile_closed_forms_on_the_gpu(bf, torch):
    n = 64
    eye = torch.eye(n, dtype=torch.float32, device="cuda")
    cu = lambda a: torch.from_numpy(a).cuda()
    ptr, idx = _lists([list(range(n))] * n)                       # complete graph with self loops
    assert np.allclose(bf.scale_profile(eye, cu(ptr), cu(idx), 3), [1, 0.125, 0.125, 0.125], rtol=1e-6)
    ptr, idx = _lists([[(i - 1) % n, i, (i + 1) % n] for i in range(n)])
    assert np.allclose(bf.scale_profile(eye, cu(ptr), cu(idx), 2), [1, 3 ** -0.5, 19 ** 0.5 / 9], rtol=1e-6)
    ptr, idx = _lists([[] for _ in range(n)])
    assert np.allclose(bf.scale_profile(eye, cu(ptr), cu(idx), 2), [1, 0, 0])
    assert np.allclose(bf.scale_profile(eye, cu(ptr), cu(idx), 0), [1])


@pytest.mark.parametrize("D,layers", [(64, 3), (37, 2), (256, 5), (600, 1)])
def test_scale_profile_matches_the_oracle(bf, torch, D, layers):
    n = 20000
    rng = np.random.default_rng(D)
    g = PowerLawGraph(n, 10.0, alpha=2.1, cap=2000, seed=D) if D != 37 else UniformGraph(n, 6, seed=2)
    indptr, indices = full_csr(g)
    noise = rng.standard_normal((n, D)).astype(np.float32)
    base = rng.standard_normal(D)
    feat = base[None, :] + 0.7 * rng.standard_normal((n, D))
    feat = (feat / np.linalg.norm(feat, axis=1, keepdims=True)).astype(np.float32)
    cu = lambda a: torch.from_numpy(a).cuda()
    dptr, dind = cu(indptr), cu(indices)
    work = torch.empty(min(layers, 2) * n * D, dtype=torch.float32, device="cuda")
    ce = bf.scale_profile(cu(noise), dptr, dind, layers, work=work)
    cf = bf.scale_profile(cu(feat), dptr, dind, layers)
    ce_want = orc.scale_profile(noise, indptr, indices, layers)
    cf_want = orc.scale_profile(feat, indptr, indices, layers)
    assert np.allclose(ce, ce_want, rtol=REL_TOL, atol=0)
    assert np.allclose(cf, cf_want, rtol=REL_TOL, atol=0)
    c_hat = (ce / ce[0]) / (cf / cf[0])
    assert (c_hat[1:] < 1).all() and (np.diff(c_hat) < 0).all()


def test_scale_profile_rejects_a_broken_graph(bf, torch):
    n, D = 100, 8
    x = torch.ones((n, D), dtype=torch.float32, device="cuda")
    ptr = torch.arange(n + 1, dtype=torch.int64, device="cuda")
    idx = torch.arange(n, dtype=torch.int64, device="cuda")
    assert np.allclose(bf.scale_profile(x, ptr, idx, 2), 8 ** 0.5)
    bad = idx.clone()
    bad[17] = n                                                   # out of range
    with pytest.raises(bf.BifeatError) as e:
        bf.scale_profile(x, ptr, bad, 2)
    assert e.value.status == -1
    with pytest.raises(bf.BifeatError):
        bf.scale_profile(x, ptr, idx, 65)
    # the library still works afterwards
    assert np.allclose(bf.scale_profile(x, ptr, idx, 1), 8 ** 0.5)


def test_two_layer_chain_replays_from_a_captured_graph(bf, torch):
    # gather_mean + aggregate_rows enqueue kernels only, so the chain can be captured and
    # replayed; rows of lists of up to 256 entries are reproduced bit for bit, rows of longer
    # lists (summed in pieces combined by atomics) to the documented bound
    N, D = 6000, 128
    spec = FeatureSpec(N, D, 9)
    _, _, s, codes = oracle_uniform_table(spec, 4)
    q = bf.Quantizer(scheme_of("uniform", 4), D)
    from bifeat_inputs.device import DeviceTable
    dcodes = gpu_build_table(q, DeviceTable(spec), N, 4096)
    rng = np.random.default_rng(3)
    ptr1, idx1 = random_csr(2000, N, 12, rng)
    ptr2, idx2 = random_csr(700, 2000, 15, rng, hubs=(900,))
    cu = lambda a: torch.from_numpy(a).cuda()
    dp1, di1, dp2, di2 = cu(ptr1), cu(idx1), cu(ptr2), cu(idx2)
    h1 = torch.empty((2000, D), dtype=torch.float32, device="cuda")
    h2 = torch.empty((700, D), dtype=torch.float32, device="cuda")
    q.gather_mean(dcodes, dp1, di1, h1)
    eager = bf.aggregate_rows(h1, dp2, di2).clone()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        q.gather_mean(dcodes, dp1, di1, h1)
        bf.aggregate_rows(h1, dp2, di2, out=h2)
    short = torch.from_numpy(np.diff(ptr2) <= 256).cuda()
    want = orc.aggregate_rows(orc.gather_mean(s, codes, ptr1, idx1), ptr2, idx2)
    for rep in range(3):
        h1.fill_(-1.0)
        h2.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(h2[short], eager[short]), f"replay {rep}"
        assert torch.allclose(h2[~short], eager[~short], rtol=1e-5, atol=1e-6), f"replay {rep}"
        assert_close(h2.cpu().numpy(), want, s, f"replay {rep} against the oracle")
        assert torch.equal(bf.aggregate_rows(h1, dp2, di2)[short], eager[short])


def _csr_from_degrees(deg, N, rng):
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    return indptr, rng.integers(0, N, int(indptr[-1])).astype(np.int64)


@pytest.mark.parametrize("case", ["threshold", "packed_longs", "long_first_and_last", "mostly_empty",
                                  "one_giant", "random_mix"])
@pytest.mark.parametrize("D", [64, 100, 7])
def test_aggregate_rows_long_list_layouts(bf, torch, case, D):
    # lists longer than 256 entries are summed in pieces by workgroups that each look after
    # 2048 consecutive entries: lengths at the threshold, long lists packed back to back
    # (as many as fit one range, with both range ends cutting a list), long lists at either
    # end of the block, long runs of empty lists, one list spanning many ranges
    rng = np.random.default_rng(len(case) * 1000 + D)
    N = 5000
    if case == "threshold":
        deg = np.array([255, 256, 257, 258, 0, 256, 257, 1, 512, 513, 2048, 2049, 2047, 3], np.int64)
    elif case == "packed_longs":
        deg = np.concatenate([[1000], np.full(40, 257), [5], np.full(17, 300), [0, 0, 2], np.full(9, 257)])
    elif case == "long_first_and_last":
        deg = np.concatenate([[3000], rng.integers(0, 12, 500), [2600]])
    elif case == "mostly_empty":
        deg = np.zeros(6000, np.int64)
        deg[[0, 1500, 1501, 5999]] = [700, 257, 4000, 300]
        deg[rng.integers(0, 6000, 200)] = 3
    elif case == "one_giant":
        deg = np.concatenate([rng.integers(0, 5, 300), [70001], rng.integers(0, 5, 300)])
    else:
        deg = np.where(rng.random(1200) < 0.05, rng.integers(257, 3000, 1200), rng.integers(0, 30, 1200))
    deg = deg.astype(np.int64)
    indptr, indices = _csr_from_degrees(deg, N, rng)
    x = (rng.standard_normal((N, D)) + 0.5).astype(np.float32)
    dx, dp, di = torch.from_numpy(x).cuda(), torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    for as_sum in (False, True):
        out = torch.full((deg.shape[0], D), 7.0, dtype=torch.float32, device="cuda")
        bf.aggregate_rows(dx, dp, di, out=out, sum=as_sum)
        _assert_rows_close(out.cpu().numpy(), orc.aggregate_rows(x, indptr, indices, sum=as_sum),
                           x, indptr, indices, as_sum, f"{case} D={D} sum={as_sum}")


@pytest.mark.timeout(600)
def test_scale_profile_at_bench_size(bf, torch):
    # the configuration `bench.py --workload mid --scale-profile 2` runs: the mid workload's
    # graph family over 2^20 nodes with self-loops, D = 100
    from bifeat_inputs import WORKLOADS
    w = WORKLOADS["mid"]
    n = 1 << 20
    g = PowerLawGraph(n, w.avg_degree, 2.1, w.cap, w.seed)
    indptr, indices = full_csr(g)
    x = feature_chunk(FeatureSpec(n, w.D, w.seed), 0, n)
    x = (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)
    dx, dp, di = torch.from_numpy(x).cuda(), torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    got = bf.scale_profile(dx, dp, di, 2)
    want = orc.scale_profile(x, indptr, indices, 2)
    assert np.allclose(got, want, rtol=REL_TOL, atol=0), (got, want)
    # one round, element by element, on a sample of destinations that includes the longest lists
    h1 = bf.aggregate_rows(dx, dp, di)
    deg = np.diff(indptr)
    sample = np.unique(np.concatenate([np.argsort(deg)[-8:], np.random.default_rng(1).integers(0, n, 300)]))
    sub_ptr = np.concatenate([[0], np.cumsum(deg[sample])]).astype(np.int64)
    sub_idx = np.concatenate([indices[indptr[v]:indptr[v + 1]] for v in sample])
    _assert_rows_close(h1[torch.from_numpy(sample).cuda()].cpu().numpy(),
                       orc.aggregate_rows(x, sub_ptr, sub_idx), x, sub_ptr, sub_idx, False, "bench size")


def test_check_lists(bf, torch):
    ptr = torch.tensor([0, 2, 2, 5], dtype=torch.int64, device="cuda")
    idx = torch.tensor([4, 0, 9, 9, 3], dtype=torch.int64, device="cuda")
    assert bf.check_lists(ptr, idx, 10)
    assert bf.check_lists(None, idx, 10)
    assert not bf.check_lists(ptr, idx, 9)                        # 9 is out of range for 9 rows
    assert not bf.check_lists(None, torch.tensor([0, -1], dtype=torch.int64, device="cuda"), 10)
    assert not bf.check_lists(torch.tensor([0, 3, 2, 5], dtype=torch.int64, device="cuda"), idx, 10)
    assert not bf.check_lists(torch.tensor([1, 2, 2, 5], dtype=torch.int64, device="cuda"), idx, 10)
    assert not bf.check_lists(torch.tensor([0, 2, 2, 4], dtype=torch.int64, device="cuda"), idx, 10)
    assert bf.check_lists(torch.zeros(1, dtype=torch.int64, device="cuda"),
                          torch.zeros(0, dtype=torch.int64, device="cuda"), 10)


@pytest.mark.parametrize("case", range(24))
def test_aggregate_rows_random(bf, torch, case):
    # seeded random shapes: width, number of rows and lists, list-length mix (empty, short,
    # a few long ones on either side of the 256-entry threshold), mean or sum
    import os
    rng = np.random.default_rng(100_000 * int(os.environ.get("BIFEAT_TEST_SEED", "0")) + 7000 + case)
    D = int(rng.choice([1, 2, 4, 5, 12, 32, 100, 128, 260, 516, 1024, 1500]))
    N = int(rng.integers(1, 3000))
    V = int(rng.integers(1, 1500))
    deg = rng.integers(0, int(rng.choice([2, 8, 40])) + 1, V)
    for _ in range(int(rng.integers(0, 6))):
        deg[rng.integers(0, V)] = int(rng.choice([255, 256, 257, 300, 1000, 2047, 2049, 5000]))
    indptr, indices = _csr_from_degrees(deg.astype(np.int64), N, rng)
    x = (rng.standard_normal((N, D)) * rng.uniform(0.01, 100) + rng.uniform(-1, 1)).astype(np.float32)
    as_sum = bool(rng.integers(0, 2))
    out = torch.full((V, D), -3.0, dtype=torch.float32, device="cuda")
    bf.aggregate_rows(torch.from_numpy(x).cuda(), torch.from_numpy(indptr).cuda(),
                      torch.from_numpy(indices).cuda(), out=out, sum=as_sum)
    _assert_rows_close(out.cpu().numpy(), orc.aggregate_rows(x, indptr, indices, sum=as_sum), x, indptr,
                       indices, as_sum, f"case {case}: D={D} N={N} V={V} sum={as_sum}")
