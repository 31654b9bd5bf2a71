"""Pins for the oracle's fp32-row aggregation and the aggregation scale factors
(Appendix A.1: later layers, C^e / C^f; Appendix A.3: C^_L; Appendix A.5: how
depth and graph structure move them)."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle as orc
from bifeat_inputs import PowerLawGraph, UniformGraph, full_csr


def _lists(rows):
    indptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int64)
    indices = np.array([j for r in rows for j in r], dtype=np.int64)
    return indptr, indices


def _transition(indptr, indices, n):
    """Dense row-normalised matrix of the lists (repeats add up)."""
    deg = np.diff(indptr)
    w = np.repeat(1.0 / np.maximum(deg, 1), deg)
    return sp.csr_matrix((w, indices, indptr), shape=(n, n)).toarray()


def _random_graph(n, max_deg, rng, self_loops=True):
    rows = []
    for i in range(n):
        nb = list(rng.integers(0, n, rng.integers(0, max_deg + 1)))
        rows.append(([i] if self_loops else []) + nb)
    return _lists(rows)


# ------------------------------------------------------------ aggregate_rows
@pytest.mark.parametrize("as_sum", [False, True])
def test_aggregate_rows_matches_sparse_matrix_product(as_sum):
    rng = np.random.default_rng(5)
    N, V, D = 300, 120, 37
    x = rng.standard_normal((N, D)).astype(np.float32)
    deg = rng.integers(0, 15, V)
    deg[0] = 0
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    indices = rng.integers(0, N, indptr[-1]).astype(np.int64)
    indices[indptr[1] + 1] = indices[indptr[1]] if deg[1] >= 2 else indices[indptr[1]]
    w = np.ones(indptr[-1]) if as_sum else np.repeat(1.0 / np.maximum(deg, 1), deg)
    want = sp.csr_matrix((w, indices, indptr), shape=(V, N)) @ x.astype(np.float64)
    got = orc.aggregate_rows(x, indptr, indices, sum=as_sum)
    assert got.dtype == np.float32 and got.shape == (V, D)
    assert np.allclose(got, want, rtol=1e-6, atol=1e-6)
    assert not got[0].any()


def test_aggregate_rows_special_cases():
    x = np.arange(12, dtype=np.float32).reshape(4, 3)
    one = orc.aggregate_rows(x, np.arange(4, dtype=np.int64), np.array([2, 0, 3], np.int64))
    assert np.array_equal(one, x[[2, 0, 3]])                     # a single neighbour is that row
    rep = orc.aggregate_rows(x, np.array([0, 3], np.int64), np.array([1, 1, 3], np.int64))
    assert np.allclose(rep, (2 * x[1] + x[3]) / 3.0)             # repeats count twice
    s = orc.aggregate_rows(x, np.array([0, 3], np.int64), np.array([1, 1, 3], np.int64), sum=True)
    assert np.array_equal(s, (2 * x[1] + x[3])[None])


def test_two_layers_are_the_squared_operator():
    rng = np.random.default_rng(6)
    n, D = 60, 9
    indptr, indices = _random_graph(n, 6, rng)
    x = rng.standard_normal((n, D)).astype(np.float32)
    P = _transition(indptr, indices, n)
    h1 = orc.aggregate_rows(x, indptr, indices)
    h2 = orc.aggregate_rows(h1, indptr, indices)
    assert np.allclose(h2, P @ P @ x.astype(np.float64), rtol=1e-5, atol=1e-6)


# ------------------------------------------------------------- scale_profile
def test_closed_forms_of_the_error_factor():
    # x = identity: row i after l rounds is row i of P^l, whose length is the exact
    # C^e_{i,l} for errors that are independent between nodes (Appendix A.1, r^e = 0)
    n = 7
    eye = np.eye(n, dtype=np.float32)
    complete = _lists([list(range(n))] * n)
    assert np.allclose(orc.scale_profile(eye, *complete, 3), [1, n ** -0.5, n ** -0.5, n ** -0.5])
    alone = _lists([[i] for i in range(n)])                      # self loop only: nothing averages out
    assert np.allclose(orc.scale_profile(eye, *alone, 4), 1.0)
    ring = _lists([[(i - 1) % n, i, (i + 1) % n] for i in range(n)])
    # one round: three weights 1/3; two rounds: weights (1,2,3,2,1)/9
    assert np.allclose(orc.scale_profile(eye, *ring, 2), [1, 3 ** -0.5, 19 ** 0.5 / 9])
    nothing = _lists([[] for _ in range(n)])
    assert np.allclose(orc.scale_profile(eye, *nothing, 2), [1, 0, 0])


def test_profile_of_identity_is_row_length_of_matrix_power():
    rng = np.random.default_rng(7)
    n = 40
    indptr, indices = _random_graph(n, 5, rng)
    P = _transition(indptr, indices, n)
    got = orc.scale_profile(np.eye(n, dtype=np.float32), indptr, indices, 4)
    want = [np.linalg.norm(np.linalg.matrix_power(P, l), axis=1).mean() for l in range(5)]
    assert np.allclose(got, want, rtol=1e-12)
    # a weighted average over at most n nodes: 1/sqrt(n) <= C <= 1, so also >= 1/n
    assert (got <= 1 + 1e-12).all() and (got >= n ** -0.5 - 1e-12).all()


def test_printed_recursion_gives_the_same_factors():
    # Appendix A.1: C_{i,l+1}^2 = sum_{j,k in N(i)} r_{l,j,k} C_{j,l} C_{k,l} / |N(i)|^2 with
    # r_{l,j,k} the correlation of the layer-l vectors of j and k.  Run it with the
    # correlations of what the profile propagates and compare the means per depth.
    rng = np.random.default_rng(8)
    n, D, L = 30, 12, 3
    indptr, indices = _random_graph(n, 4, rng)
    x = rng.standard_normal((n, D))
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    P = _transition(indptr, indices, n)
    Cf = np.ones(n)
    h = x.copy()
    means = [1.0]
    for _ in range(L):
        norms = np.linalg.norm(h, axis=1)
        r = (h @ h.T) / np.outer(norms, norms)
        nxt = np.empty(n)
        for i in range(n):
            nb = indices[indptr[i]:indptr[i + 1]]
            nxt[i] = np.sqrt(sum(r[j, k] * Cf[j] * Cf[k] for j in nb for k in nb)) / len(nb)
        Cf, h = nxt, P @ h
        means.append(Cf.mean())
    got = orc.scale_profile(x.astype(np.float32), indptr, indices, L)
    assert np.allclose(got, means, rtol=1e-6)


def test_noise_run_estimates_the_exact_error_factor():
    rng = np.random.default_rng(9)
    n, D = 50, 4096
    indptr, indices = _random_graph(n, 6, rng)
    P = _transition(indptr, indices, n)
    e = rng.standard_normal((n, D)).astype(np.float32)
    s = orc.scale_profile(e, indptr, indices, 3)
    est = s / s[0]
    exact = [np.linalg.norm(np.linalg.matrix_power(P, l), axis=1).mean() for l in range(4)]
    assert abs(s[0] / np.sqrt(D) - 1) < 0.01
    assert np.allclose(est, exact, rtol=0.03)


def test_feature_factor_and_the_ratio():
    rng = np.random.default_rng(10)
    n, D, L = 80, 64, 3
    indptr, indices = _random_graph(n, 8, rng)
    same = np.tile(rng.standard_normal(D), (n, 1))
    same /= np.linalg.norm(same, axis=1, keepdims=True)
    assert np.allclose(orc.scale_profile(same.astype(np.float32), indptr, indices, L), 1.0, rtol=1e-6)
    # positively correlated unit rows keep more of their length than independent errors:
    # C^e <= C^f, so C^_L <= 1, and both shrink with depth
    x = same + 0.5 * rng.standard_normal((n, D)) / np.sqrt(D)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    cf = orc.scale_profile(x.astype(np.float32), indptr, indices, L)
    ce = orc.scale_profile(np.eye(n, dtype=np.float32), indptr, indices, L)
    assert (ce[1:] < cf[1:]).all()
    assert (np.diff(ce) < 0).all() and (np.diff(cf) <= 1e-9).all()
    c_hat = ce / cf
    assert (np.diff(c_hat) < 0).all()                            # deeper models tolerate more error


def test_hub_graphs_keep_more_of_the_error_than_uniform_ones():
    # Appendix A.5: with the same number of edges, lists dominated by a few
    # high-degree nodes cancel less of the error than evenly spread ones
    n = 400
    hubs = PowerLawGraph(n, 8.0, alpha=2.1, cap=200, seed=1)
    even = UniformGraph(n, 8, seed=1)
    eye = np.eye(n, dtype=np.float32)
    ce_h = orc.scale_profile(eye, *full_csr(hubs), 2)
    ce_u = orc.scale_profile(eye, *full_csr(even), 2)
    assert ce_h[2] > 1.5 * ce_u[2]
    # and a denser graph of the same kind cancels more
    ce_d = orc.scale_profile(eye, *full_csr(UniformGraph(n, 24, seed=1)), 2)
    assert ce_d[2] < ce_u[2]
