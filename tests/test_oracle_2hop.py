"""Pins for the oracle's two-round aggregation straight from the packed table
(Appendix A.1 applied twice: the mean over the seed block of the means over the
outer block)."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk


def _quantized(rows=500, D=20, bits=4, seed=21):
    x = feature_chunk(FeatureSpec(rows, D, seed), 0, rows)
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, bits)
    codes = orc.pack(orc.uniform_encode(x, bits, mn, inv), bits)
    return x, orc.Scheme.uniform(mn, scale, bits), codes


def _csr(V, N, max_deg, rng, empty=(0,)):
    deg = rng.integers(1, max_deg + 1, V)
    for e in empty:
        deg[e] = 0
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    indices = rng.integers(0, N, indptr[-1]).astype(np.int64)
    return indptr, indices


def _row_stochastic(indptr, indices, ncols):
    deg = np.diff(indptr)
    w = np.repeat(1.0 / np.maximum(deg, 1), deg)
    return sp.csr_matrix((w, indices, indptr), shape=(len(indptr) - 1, ncols))   # repeats add up


def test_hand_counted_example():
    # 8-bit codes with min 0 and max 255 decode to the code itself (scale 1).
    # rows: r0 = (10, 20), r1 = (30, 40), r2 = (50, 0), r3 = (2, 4)
    D = 2
    q = np.array([[10, 20], [30, 40], [50, 0], [2, 4]], np.int64)
    s = orc.Scheme.uniform(np.zeros(D, np.float32), np.ones(D, np.float32), 8)
    codes = orc.pack(q, 8)
    # outer block: u0 = {r0, r1} -> (20, 30); u1 = {} -> 0 (counts below); u2 = {r2, r2, r3} -> (34, 4/3)
    indptr1 = np.array([0, 2, 2, 5], np.int64)
    indices1 = np.array([0, 1, 2, 2, 3], np.int64)
    # seed block: v0 = {u0, u2} -> (27, 47/3); v1 = {u1, u0} -> (10, 15); v2 = {}; v3 = {u2, u2, u0, u1}
    indptr2 = np.array([0, 2, 4, 4, 8], np.int64)
    indices2 = np.array([0, 2, 1, 0, 2, 2, 0, 1], np.int64)
    got = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
    want = np.array([[27.0, 47.0 / 3.0], [10.0, 15.0], [0.0, 0.0],
                     [(34 + 34 + 20 + 0) / 4.0, (4 / 3 + 4 / 3 + 30 + 0) / 4.0]])
    assert np.array_equal(got, want.astype(np.float32))


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_matches_product_of_row_stochastic_matrices(bits):
    x, s, codes = _quantized(bits=bits)
    rng = np.random.default_rng(100 + bits)
    N, V1, V2 = x.shape[0], 90, 30
    indptr1, indices1 = _csr(V1, N, 9, rng, empty=(0, 17))
    indptr2, indices2 = _csr(V2, V1, 7, rng, empty=(3,))
    indices2[indptr2[5]] = 0                                   # a seed that lists an empty outer list
    got = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
    dec = orc.gather_dequant(s, codes, np.arange(N)).astype(np.float64)
    want = _row_stochastic(indptr2, indices2, V1) @ (_row_stochastic(indptr1, indices1, N) @ dec)
    assert np.allclose(got, want, rtol=1e-6, atol=1e-7)
    assert not got[3].any()


def test_log_and_vq_tables():
    x = feature_chunk(FeatureSpec(400, 16, 5), 0, 400)
    rng = np.random.default_rng(9)
    indptr1, indices1 = _csr(60, 400, 8, rng)
    indptr2, indices2 = _csr(25, 60, 6, rng)
    A = _row_stochastic(indptr2, indices2, 60) @ _row_stochastic(indptr1, indices1, 400)
    e_min, e_max = orc.log_range(orc.log_fit(x))
    T, V = orc.log_tables(e_min, e_max, 2)
    s = orc.Scheme.log(16, V, 2)
    codes = orc.pack(orc.log_encode(x, 2, T), 2)
    dec = orc.gather_dequant(s, codes, np.arange(400)).astype(np.float64)
    assert np.allclose(orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2), A @ dec,
                       rtol=1e-6, atol=1e-7)
    cb, _ = orc.vq_train(x, 4, 16, iters=3)
    s = orc.Scheme.vq(16, cb)
    codes = orc.pack(orc.vq_assign(x, 4, cb), 8)
    dec = orc.gather_dequant(s, codes, np.arange(400)).astype(np.float64)
    assert np.allclose(orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2), A @ dec,
                       rtol=1e-6, atol=1e-7)


def test_reduces_to_one_round_and_to_the_chain():
    x, s, codes = _quantized()
    rng = np.random.default_rng(3)
    N, V1 = x.shape[0], 70
    indptr1, indices1 = _csr(V1, N, 11, rng)
    # seed lists of exactly one entry: the second round is a row selection
    pick = rng.integers(0, V1, 40).astype(np.int64)
    one = orc.gather_mean_2hop(s, codes, indptr1, indices1, np.arange(41, dtype=np.int64), pick)
    assert np.array_equal(one, orc.gather_mean(s, codes, indptr1, indices1)[pick])
    # outer lists of exactly one entry: the first round is a decode
    rows = rng.integers(0, N, V1).astype(np.int64)
    indptr2, indices2 = _csr(30, V1, 6, rng)
    two = orc.gather_mean_2hop(s, codes, np.arange(V1 + 1, dtype=np.int64), rows, indptr2, indices2)
    assert np.array_equal(two, orc.gather_mean(s, codes, indptr2, rows[indices2]))
    # general lists: the chain of the two one-round calls rounds g1 to fp32 in between
    chain = orc.aggregate_rows(orc.gather_mean(s, codes, indptr1, indices1), indptr2, indices2)
    got = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
    assert np.allclose(got, chain, rtol=3e-7, atol=1e-7)


def test_constant_rows_average_to_the_constant():
    x, s, codes = _quantized()
    rng = np.random.default_rng(4)
    indptr1, _ = _csr(20, 500, 5, rng, empty=())
    indptr2, indices2 = _csr(10, 20, 4, rng, empty=())
    indices1 = np.full(indptr1[-1], 123, np.int64)
    got = orc.gather_mean_2hop(s, codes, indptr1, indices1, indptr2, indices2)
    row = orc.gather_dequant(s, codes, np.array([123]))
    assert np.allclose(got, np.repeat(row, 10, 0), rtol=2e-7)
