"""Pins for the oracle's gather / decode / neighbourhood mean (Sec. 3.3, Appendix A.1)."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk


def _quantized(rows=600, D=20, bits=4, seed=11):
    x = feature_chunk(FeatureSpec(rows, D, seed), 0, rows)
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, bits)
    codes = orc.pack(orc.uniform_encode(x, bits, mn, inv), bits)
    return x, orc.Scheme.uniform(mn, scale, bits), codes


def _random_csr(V, N, max_deg, rng):
    deg = rng.integers(0, max_deg + 1, V)
    deg[0] = 0                                               # an empty neighbourhood
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    indices = rng.integers(0, N, indptr[-1]).astype(np.int64)
    if deg[1] >= 2:
        indices[indptr[1] + 1] = indices[indptr[1]]          # a repeated neighbour
    return indptr, indices


def test_gather_codes_is_row_indexing():
    _, _, codes = _quantized()
    idx = np.array([5, 0, 599, 5, 17], np.int64)
    assert np.array_equal(orc.gather_codes(codes, idx), codes[idx])
    assert orc.gather_codes(codes, np.zeros(0, np.int64)).shape == (0, codes.shape[1])


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_mean_matches_sparse_matrix_product(bits):
    x, s, codes = _quantized(bits=bits)
    rng = np.random.default_rng(bits)
    indptr, indices = _random_csr(150, x.shape[0], 12, rng)
    got = orc.gather_mean(s, codes, indptr, indices)
    dec = orc.gather_dequant(s, codes, np.arange(x.shape[0])).astype(np.float64)
    deg = np.diff(indptr)
    w = np.repeat(1.0 / np.maximum(deg, 1), deg)
    A = sp.csr_matrix((w, indices, indptr), shape=(150, x.shape[0]))   # duplicates sum up
    want = A @ dec
    assert np.allclose(got, want, rtol=1e-6, atol=1e-6)
    assert not got[0].any()                                  # empty list -> zero row


def test_single_neighbour_is_that_row_and_constant_rows_average_to_constant():
    x, s, codes = _quantized()
    idx = np.array([3, 77, 401], np.int64)
    one = orc.gather_mean(s, codes, np.arange(4, dtype=np.int64), idx)
    assert np.array_equal(one, orc.gather_dequant(s, codes, idx))
    same = orc.gather_mean(s, codes, np.array([0, 7], np.int64), np.full(7, 42, np.int64))
    assert np.allclose(same, orc.gather_dequant(s, codes, np.array([42])), rtol=1e-7)


def test_mean_for_log_and_vq_tables_matches_sparse_product():
    x = feature_chunk(FeatureSpec(500, 16, 13), 0, 500)
    rng = np.random.default_rng(0)
    indptr, indices = _random_csr(80, 500, 9, rng)
    deg = np.diff(indptr)
    A = sp.csr_matrix((np.repeat(1.0 / np.maximum(deg, 1), deg), indices, indptr), shape=(80, 500))
    e_min, e_max = orc.log_range_clipped(x, 0.01)
    T, V = orc.log_tables(e_min, e_max, 4)
    s = orc.Scheme.log(16, V, 4)
    codes = orc.pack(orc.log_encode(x, 4, T), 4)
    dec = orc.gather_dequant(s, codes, np.arange(500)).astype(np.float64)
    assert np.allclose(orc.gather_mean(s, codes, indptr, indices), A @ dec, rtol=1e-6, atol=1e-6)
    cb, _ = orc.vq_train(x, 4, 16, iters=3)
    s = orc.Scheme.vq(16, cb)
    codes = orc.pack(orc.vq_assign(x, 4, cb), 8)
    dec = orc.gather_dequant(s, codes, np.arange(500)).astype(np.float64)
    assert np.allclose(orc.gather_mean(s, codes, indptr, indices), A @ dec, rtol=1e-6, atol=1e-6)


def test_rounding_errors_cancel_under_averaging():
    # independent per-row rounding errors (Assumption 1): the error of a mean
    # over n distinct rows has RMS ~ per-row RMS / sqrt(n)  (Appendix A.1, the
    # C^e recursion with zero cross-correlation)
    rows, D, n = 40000, 8, 16
    x, s, codes = _quantized(rows, D, bits=4)
    V = rows // n
    indptr = np.arange(V + 1, dtype=np.int64) * n
    indices = np.random.default_rng(0).permutation(rows).astype(np.int64)
    mean_q = orc.gather_mean(s, codes, indptr, indices).astype(np.float64)
    mean_x = x[indices].reshape(V, n, D).astype(np.float64).mean(1)
    dec = orc.gather_dequant(s, codes, np.arange(rows)).astype(np.float64)
    rms_row = np.sqrt(((dec - x) ** 2).mean(0))
    rms_mean = np.sqrt(((mean_q - mean_x) ** 2).mean(0))
    assert np.allclose(rms_mean, rms_row / np.sqrt(n), rtol=0.1)


# ------------------------------------------- other aggregators over the same compressed rows
@pytest.mark.parametrize("bits", [1, 4])
def test_sum_matches_sparse_matrix_product(bits):
    x, s, codes = _quantized(bits=bits)
    rng = np.random.default_rng(40 + bits)
    indptr, indices = _random_csr(150, x.shape[0], 12, rng)
    got = orc.gather_sum(s, codes, indptr, indices)
    dec = orc.gather_dequant(s, codes, np.arange(x.shape[0])).astype(np.float64)
    A = sp.csr_matrix((np.ones(len(indices)), indices, indptr), shape=(150, x.shape[0]))
    want = A @ dec                                           # repeats add up in the CSR product
    assert np.allclose(got, want, rtol=1e-6, atol=1e-6)
    assert not got[0].any()
    # mean = sum / count wherever the list is not empty
    n = np.diff(indptr)[:, None]
    mean = orc.gather_mean(s, codes, indptr, indices)
    assert np.allclose(mean[n[:, 0] > 0], (got / np.maximum(n, 1))[n[:, 0] > 0], rtol=1e-6, atol=1e-7)


def test_mean_with_self_in_the_list_is_the_self_loop_normalisation():
    # Appendix A.1 writes the layer with D^-1 (A + I): listing v among its own
    # neighbours turns the plain mean into that operator
    x, s, codes = _quantized(rows=300)
    rng = np.random.default_rng(77)
    N = x.shape[0]
    deg = rng.integers(0, 9, N)
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    indices = rng.integers(0, N, indptr[-1]).astype(np.int64)
    # lists with the destination itself appended
    ptr2 = indptr + np.arange(N + 1)
    idx2 = np.empty(ptr2[-1], np.int64)
    for v in range(N):
        idx2[ptr2[v]:ptr2[v + 1] - 1] = indices[indptr[v]:indptr[v + 1]]
        idx2[ptr2[v + 1] - 1] = v
    got = orc.gather_mean(s, codes, ptr2, idx2)
    dec = orc.gather_dequant(s, codes, np.arange(N)).astype(np.float64)
    A = sp.csr_matrix((np.ones(len(indices)), indices, indptr), shape=(N, N)) + sp.identity(N)
    want = sp.diags(1.0 / np.asarray(A.sum(1)).ravel()) @ (A @ dec)
    assert np.allclose(got, want, rtol=1e-6, atol=1e-7)
