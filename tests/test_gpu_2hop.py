"""GPU parity for two rounds of the neighbourhood mean straight from the packed table
(Appendix A.1 applied twice; bifeat_gather_mean_2hop) against the CPU oracle: both kernels
(the register-accumulator form under the caller's bound on the list lengths, the general
form without it), every kind of code, ragged shapes, the degenerate lists, and the broken
promise."""
import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import FeatureSpec, PowerLawGraph, draw_seeds, feature_chunk, sample_blocks
from helpers import assert_close, oracle_uniform_table, scheme_of

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bf():
    import paper_2207_14696_amd as m
    m.load_library()
    return m


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


def _table(bf, kind, bits, D, N=6000, seed=7, w=0, length=0):
    """Oracle-made packed table, its oracle scheme, and a quantizer with the same parameters."""
    spec = FeatureSpec(N, D, seed)
    x = feature_chunk(spec, 0, N)
    if kind == "uniform":
        _, (mn, mx, _, _), s, codes = oracle_uniform_table(spec, bits)
        q = bf.Quantizer(scheme_of("uniform", bits), D)
        q.params_set_uniform(mn, mx)
    elif kind == "log":
        e_min, e_max = orc.log_range(orc.log_fit(x))
        T, Vt = orc.log_tables(e_min, e_max, bits)
        codes = orc.pack(orc.log_encode(x, bits, T), bits)
        s = orc.Scheme.log(D, Vt, bits)
        q = bf.Quantizer(scheme_of("log", bits), D)
        q.params_set_log(e_min, e_max)
    else:
        cb, _ = orc.vq_train(x[:2000], w, length, iters=2)
        codes = orc.pack(orc.vq_assign(x, w, cb), 8)
        s = orc.Scheme.vq(D, cb)
        q = bf.Quantizer(scheme_of("vq", 8, w, length), D)
        q.params_set_codebooks(cb)
    assert codes.shape[1] == q.row_bytes
    return s, codes, q


def _blocks(N, V1, V2, max1, max2, rng):
    """Outer lists of table rows and seed lists of outer destinations: ragged lengths, empty
    lists in both blocks, a seed entry that names an empty outer list, repeats."""
    d1 = rng.integers(0, max1 + 1, V1)
    d1[0] = 0
    d1[1] = max1
    indptr1 = np.concatenate([[0], np.cumsum(d1)]).astype(np.int64)
    indices1 = rng.integers(0, N, int(indptr1[-1])).astype(np.int64)
    d2 = rng.integers(0, max2 + 1, V2)
    d2[0] = 0
    d2[1] = max2
    indptr2 = np.concatenate([[0], np.cumsum(d2)]).astype(np.int64)
    indices2 = rng.integers(0, V1, int(indptr2[-1])).astype(np.int64)
    indices2[indptr2[1]] = 0                               # the empty outer list, listed
    indices2[indptr2[1] + 1] = indices2[indptr2[1] + 2]    # a repeated entry
    return indptr1, indices1, indptr2, indices2


CASES = [("uniform", 4, 768), ("uniform", 4, 100), ("uniform", 4, 128), ("uniform", 1, 768),
         ("uniform", 1, 128), ("uniform", 2, 128), ("uniform", 2, 52), ("uniform", 8, 128),
         ("uniform", 8, 36), ("uniform", 4, 2048), ("log", 1, 64), ("log", 2, 128), ("log", 2, 100),
         ("log", 4, 64), ("uniform", 4, 30)]


@pytest.mark.parametrize("hint", [0, 12, 25, 64])
@pytest.mark.parametrize("kind,bits,D", CASES)
def test_matches_the_oracle(bf, torch, kind, bits, D, hint):
    s, codes, q = _table(bf, kind, bits, D, N=3000 if D >= 768 else 6000)
    rng = np.random.default_rng(1000 * bits + D + hint)
    m = hint if hint else 40
    V1, V2 = 701, 203
    indptr1, indices1, indptr2, indices2 = _blocks(codes.shape[0], V1, V2, m, min(m, 25), rng)
    want = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if hint:
        q.set_option("mean_max_degree", hint)
    got = q.gather_mean_2hop(cu(codes), cu(indptr1), cu(indices1), cu(indptr2), cu(indices2))
    assert q.poll_status(wait=True)
    got = got.cpu().numpy()
    assert_close(got, want, s, f"{kind} {bits}-bit D={D} hint={hint}")
    assert not got[0].any()


def test_vector_codes_and_wide_tables_take_the_general_kernel(bf, torch):
    rng = np.random.default_rng(5)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for kind, bits, D, w, length in [("vq", 8, 64, 8, 16), ("vq", 8, 30, 5, 8), ("uniform", 8, 4096, 0, 0)]:
        s, codes, q = _table(bf, kind, bits, D, N=2500, w=w, length=length)
        q.set_option("mean_max_degree", 16)
        indptr1, indices1, indptr2, indices2 = _blocks(codes.shape[0], 300, 90, 16, 9, rng)
        want = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
        got = q.gather_mean_2hop(cu(codes), cu(indptr1), cu(indices1), cu(indptr2), cu(indices2)).cpu().numpy()
        assert_close(got, want, s, f"{kind} D={D}")


def test_long_lists_without_a_bound(bf, torch):
    # hubs in both blocks: lists of hundreds of entries, far beyond the short-list form
    s, codes, q = _table(bf, "uniform", 4, 128)
    rng = np.random.default_rng(8)
    V1, V2 = 400, 60
    d1 = rng.integers(0, 12, V1)
    d1[[3, 50]] = [900, 2500]
    indptr1 = np.concatenate([[0], np.cumsum(d1)]).astype(np.int64)
    indices1 = rng.integers(0, codes.shape[0], int(indptr1[-1])).astype(np.int64)
    d2 = rng.integers(0, 9, V2)
    d2[5] = 700
    indptr2 = np.concatenate([[0], np.cumsum(d2)]).astype(np.int64)
    indices2 = rng.integers(0, V1, int(indptr2[-1])).astype(np.int64)
    indices2[indptr2[5]:indptr2[5] + 2] = [3, 50]
    want = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
    cu = lambda a: torch.from_numpy(a).cuda()
    got = q.gather_mean_2hop(cu(codes), cu(indptr1), cu(indices1), cu(indptr2), cu(indices2)).cpu().numpy()
    assert_close(got, want, s, "hubs")


@pytest.mark.parametrize("hint", [0, 10])
def test_edge_cases(bf, torch, hint):
    s, codes, q = _table(bf, "uniform", 4, 128)
    if hint:
        q.set_option("mean_max_degree", hint)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dcodes = cu(codes)
    i64 = lambda *a: cu(np.array(a, dtype=np.int64))
    none = cu(np.zeros(0, np.int64))
    # no seeds at all
    assert q.gather_mean_2hop(dcodes, i64(0, 2), i64(4, 5), i64(0), none).shape == (0, 128)
    # every seed list empty, no outer block: zero rows, written
    out = torch.ones((3, 128), dtype=torch.float32, device="cuda")
    q.gather_mean_2hop(dcodes, i64(0), none, i64(0, 0, 0, 0), none, out=out)
    assert not out.cpu().numpy().any()
    # one entry per list in both blocks: a plain decode, bit for bit
    rows = np.array([17, 0, 5999, 17], np.int64)
    got = q.gather_mean_2hop(dcodes, cu(np.arange(5, dtype=np.int64)), cu(rows),
                             cu(np.arange(4, dtype=np.int64)), i64(3, 1, 2))
    assert np.array_equal(got.cpu().numpy(), orc.gather_dequant(s, codes, rows[[3, 1, 2]]))
    # seed lists that name only empty outer lists: zero rows
    got = q.gather_mean_2hop(dcodes, i64(0, 0, 2), i64(1, 2), i64(0, 2, 3), i64(0, 0, 1)).cpu().numpy()
    assert not got[0].any()
    assert_close(got[1:2], orc.gather_mean(s, codes, np.array([0, 2]), np.array([1, 2])), s, "one outer list")
    assert q.poll_status(wait=True)


def test_a_list_beyond_the_promised_bound_gives_nan_rows_and_raises_the_status(bf, torch):
    s, codes, q = _table(bf, "uniform", 4, 128)
    q.set_option("mean_max_degree", 8)
    rng = np.random.default_rng(2)
    indptr1, indices1, indptr2, indices2 = _blocks(codes.shape[0], 120, 40, 8, 8, rng)
    # outer list 7 grows to 9 entries; seeds that list it break the promise, the others do not
    extra = rng.integers(0, codes.shape[0], 9).astype(np.int64)
    d1 = np.diff(indptr1)
    indices1 = np.concatenate([indices1[:indptr1[7]], extra, indices1[indptr1[8]:]])
    d1[7] = 9
    indptr1 = np.concatenate([[0], np.cumsum(d1)]).astype(np.int64)
    indices2[indptr2[4]] = 7
    want = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    got = q.gather_mean_2hop(cu(codes), cu(indptr1), cu(indices1), cu(indptr2), cu(indices2)).cpu().numpy()
    hit = np.array([(indices2[indptr2[v]:indptr2[v + 1]] == 7).any() for v in range(40)])
    assert hit[4] and np.isnan(got[hit]).all()
    assert_close(got[~hit], want[~hit], s, "rows that kept the promise")
    assert not q.poll_status(wait=True)          # raised ...
    assert q.poll_status(wait=True)              # ... and cleared by the look
    # a seed list that is itself too long
    q2 = _table(bf, "uniform", 4, 128)[2]
    q2.set_option("mean_max_degree", 3)
    got = q2.gather_mean_2hop(cu(codes), cu(np.arange(6, dtype=np.int64)), cu(np.arange(5, dtype=np.int64)),
                              cu(np.array([0, 4, 5], np.int64)), cu(np.array([0, 1, 2, 3, 4], np.int64))).cpu().numpy()
    assert np.isnan(got[0]).all()
    assert np.array_equal(got[1], orc.gather_dequant(s, codes, np.array([4]))[0])
    assert not q2.poll_status(wait=True)


@pytest.mark.parametrize("kind,bits,D,fanouts", [("uniform", 4, 100, [25, 10]), ("uniform", 2, 128, [10, 5]),
                                                 ("uniform", 4, 768, [25, 15]), ("log", 2, 128, [10, 5])])
def test_sampled_minibatch_blocks_and_the_chain(bf, torch, kind, bits, D, fanouts):
    # the blocks a sampler hands over: seed lists renumbered to the outer block's destinations;
    # the fused call against the oracle and against the library's own two-call chain
    N = 20000
    s, codes, q = _table(bf, kind, bits, D, N=N, seed=3)
    g = PowerLawGraph(N, 12.0, seed=5)
    seeds = draw_seeds(g, 1024, 5, 0)
    blocks, _ = sample_blocks(g, seeds, fanouts, 5, 0)
    inner, outer = blocks[0], blocks[1]
    local = np.searchsorted(outer.dst, inner.indices)
    want = orc.gather_mean_2hop(s, codes, outer.indptr, outer.indices, inner.indptr, local)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dcodes, p1, i1, p2, i2 = cu(codes), cu(outer.indptr), cu(outer.indices), cu(inner.indptr), cu(local)
    chain = bf.aggregate_rows(q.gather_mean(dcodes, p1, i1), p2, i2).cpu().numpy()
    plain = q.gather_mean_2hop(dcodes, p1, i1, p2, i2).cpu().numpy()
    q.set_option("mean_max_degree", max(fanouts))
    fused = q.gather_mean_2hop(dcodes, p1, i1, p2, i2).cpu().numpy()
    assert q.poll_status(wait=True)
    assert_close(plain, want, s, "general kernel")
    assert_close(fused, want, s, "bounded kernel")
    A = np.abs(orc.gather_dequant(s, codes, np.arange(N))).max(axis=0).astype(np.float64)[None, :]
    assert (np.abs(fused.astype(np.float64) - chain) <= 2e-5 * np.maximum(np.abs(chain), A)).all()


def test_random_shapes_bounds_and_row_strides(bf, torch):
    # lane geometries of the bounded kernel: rows of 16 bytes to 1 KB (1 to 64 lanes per row, one
    # to sixteen groups per seed), bounds from 1 to 64, seed counts that leave ragged tiles, both
    # row strides; every element against the oracle
    rng = np.random.default_rng(2024)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for case in range(48):
        bits = int(rng.choice([1, 2, 4, 8]))
        D = 4 * int(rng.integers(1, {1: 512, 2: 256, 4: 256, 8: 96}[bits] + 1))
        kind = "log" if bits <= 2 and rng.random() < 0.4 else "uniform"
        m = int(rng.choice([1, 2, 3, 7, 15, 16, 17, 18, 31, 32, 33, 48, 64]))
        align = int(rng.choice([16, 128]))
        N = int(rng.integers(200, 1500))
        spec = FeatureSpec(N, D, 100 + case)
        x = feature_chunk(spec, 0, N)
        if kind == "uniform":
            _, (mn, mx, _, _), s, codes = oracle_uniform_table(spec, bits)
            q = bf.Quantizer(scheme_of("uniform", bits), D, row_align=align)
            q.params_set_uniform(mn, mx)
        else:
            e_min, e_max = orc.log_range(orc.log_fit(x))
            T, Vt = orc.log_tables(e_min, e_max, bits)
            codes = orc.pack(orc.log_encode(x, bits, T), bits)
            s = orc.Scheme.log(D, Vt, bits)
            q = bf.Quantizer(scheme_of("log", bits), D, row_align=align)
            q.params_set_log(e_min, e_max)
        table = np.zeros((N, q.row_bytes), np.uint8)           # the library's row stride, payload first
        table[:, :codes.shape[1]] = codes
        V1, V2 = int(rng.integers(1, 400)), int(rng.integers(1, 300))
        d1 = rng.integers(0, m + 1, V1)
        d2 = rng.integers(0, m + 1, V2)
        if rng.random() < 0.5:
            d2 = np.minimum(d2, rng.integers(1, 6))            # short seed lists: few groups per seed
        indptr1 = np.concatenate([[0], np.cumsum(d1)]).astype(np.int64)
        indices1 = rng.integers(0, N, int(indptr1[-1])).astype(np.int64)
        indptr2 = np.concatenate([[0], np.cumsum(d2)]).astype(np.int64)
        indices2 = rng.integers(0, V1, int(indptr2[-1])).astype(np.int64)
        want = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
        q.set_option("mean_max_degree", m)
        got = q.gather_mean_2hop(cu(table), cu(indptr1), cu(indices1), cu(indptr2), cu(indices2))
        assert q.poll_status(wait=True), f"case {case}"
        assert_close(got.cpu().numpy(), want, s, f"case {case}: {kind} {bits}-bit D={D} m={m} stride {q.row_bytes}")


@pytest.mark.parametrize("D,w,length", [(64, 8, 16), (96, 4, 32), (128, 16, 64), (768, 8, 256), (40, 8, 8),
                                        (192, 4, 16)])   # 48 parts in slices of 32: a slice with idle lanes
def test_vector_codes_with_the_codebooks_on_chip(bf, torch, D, w, length):
    # power-of-two widths take the kernel that keeps codebook slices in LDS: short and long lists,
    # empty ones, repeats; with and without a bound (it needs none)
    s, codes, q = _table(bf, "vq", 8, D, N=3000, w=w, length=length)
    rng = np.random.default_rng(D + w)
    V1, V2 = 500, 131
    indptr1, indices1, indptr2, indices2 = _blocks(codes.shape[0], V1, V2, 12, 9, rng)
    d1 = np.diff(indptr1)
    d1[7] = 150                                             # one long outer list
    indptr1 = np.concatenate([[0], np.cumsum(d1)]).astype(np.int64)
    indices1 = rng.integers(0, codes.shape[0], int(indptr1[-1])).astype(np.int64)
    indices2[indptr2[1] + 3] = 7
    want = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    args = (cu(codes), cu(indptr1), cu(indices1), cu(indptr2), cu(indices2))
    got = q.gather_mean_2hop(*args).cpu().numpy()
    assert_close(got, want, s, f"vq D={D} w={w}")
    assert not got[0].any()
    # the one-round call over the outer block shares the slice geometry
    assert_close(q.gather_mean(args[0], args[1], args[2]).cpu().numpy(),
                 orc.gather_mean(s, codes, indptr1, indices1), s, f"vq D={D} w={w} one round")
    q.set_option("vq_sliced", 0)                            # the same from L2 (general kernel)
    assert_close(q.gather_mean_2hop(*args).cpu().numpy(), want, s, f"vq D={D} w={w} from L2")


def test_replays_from_a_captured_graph(bf, torch):
    # scalar codes: the call only enqueues kernels; vector codes: the workspace is sized before
    # the capture, and a capture that would need a larger one runs the kernel that needs none
    rng = np.random.default_rng(77)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for kind, bits, D, w, length, hint in [("uniform", 4, 128, 0, 0, 12), ("uniform", 2, 64, 0, 0, 0),
                                           ("vq", 8, 64, 8, 16, 0)]:
        s, codes, q = _table(bf, kind, bits, D, N=3000, w=w, length=length)
        small = _blocks(codes.shape[0], 300, 90, 12, 9, rng)
        big = _blocks(codes.shape[0], 2500, 700, 12, 9, rng)
        dcodes = cu(codes)
        d_small, d_big = [cu(a) for a in small], [cu(a) for a in big]
        out_small = torch.empty((90, D), device="cuda")
        out_big = torch.empty((700, D), device="cuda")
        q.set_option("mean_max_degree", hint)
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            q.gather_mean_2hop(dcodes, *d_small, out=out_small)       # sizes the workspace (vector codes)
            stream.synchronize()
            g_small, g_big = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_small, stream=stream):
                q.gather_mean_2hop(dcodes, *d_small, out=out_small)
            with torch.cuda.graph(g_big, stream=stream):
                q.gather_mean_2hop(dcodes, *d_big, out=out_big)
        want_small = orc.gather_mean_2hop(s, codes, *small)
        want_big = orc.gather_mean_2hop(s, codes, *big)
        for rep in range(3):
            out_small.fill_(float("nan"))
            out_big.fill_(float("nan"))
            g_small.replay()
            g_big.replay()
            torch.cuda.synchronize()
            assert_close(out_small.cpu().numpy(), want_small, s, f"{kind}: captured small, replay {rep}")
            assert_close(out_big.cpu().numpy(), want_big, s, f"{kind}: captured big, replay {rep}")
            if rep == 0:   # eager work (and workspace growth) between replays
                got = q.gather_mean_2hop(dcodes, *d_big)
                assert_close(got.cpu().numpy(), want_big, s, f"{kind}: eager between replays")
        q.set_option("mean_max_degree", 0)
        assert q.poll_status()
