"""Pins for the oracle's vector codes (Sec. 3.2, Appendix D)."""
import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk


def _table(rows=1500, D=24, seed=7):
    return feature_chunk(FeatureSpec(rows, D, seed), 0, rows)


def test_compression_ratio_bytes():
    # CR = width * 32 / log2(length) (Sec. 3.2): width 8, length 256 -> 32
    s = orc.Scheme.vq(768, np.zeros((96, 256, 8), np.float32))
    assert s.row_bytes == 96 and 768 * 4 / s.row_bytes == 8 * 32 / np.log2(256) == 32


@pytest.mark.parametrize("w,length", [(8, 256), (4, 16), (5, 7), (1, 4)])
def test_assign_is_bruteforce_nearest(w, length):
    x = _table()
    D = x.shape[1]
    P = orc.vq_parts(D, w)
    rng = np.random.default_rng(w)
    cb = rng.normal(size=(P, length, w)).astype(np.float32)
    q = orc.vq_assign(x, w, cb)
    xp = np.zeros((x.shape[0], P * w))
    xp[:, :D] = x                                            # short last part zero-padded
    for p in range(P):
        sub = xp[:, p * w:(p + 1) * w]
        d2 = ((sub[:, None, :] - cb[p].astype(np.float64)[None, :, :]) ** 2).sum(-1)
        best = d2.argmin(1)
        same = best == q[:, p]
        assert same.mean() > 0.999
        # where they differ it is a rounding-level tie
        rows = np.nonzero(~same)[0]
        assert np.allclose(d2[rows, best[rows]], d2[rows, q[rows, p]], rtol=1e-5)


def test_ties_go_to_lowest_index():
    cb = np.zeros((1, 4, 2), np.float32)
    cb[0, 1] = cb[0, 2] = [1, 1]                             # entries 1 and 2 identical
    q = orc.vq_assign(np.array([[1, 1], [0, 0], [0.9, 1.2]], np.float32), 2, cb)
    assert list(q[:, 0]) == [1, 0, 1]


def test_lloyd_distortion_never_increases():
    x = _table()
    _, dist = orc.vq_train(x, 8, 32, iters=10)
    assert np.all(np.diff(dist) <= 1e-9 * dist[0]) and dist[-1] < dist[0]


def test_codebook_as_large_as_the_data_is_lossless():
    x = _table(40, 12)
    cb, dist = orc.vq_train(x, 4, 64, iters=3)
    q = orc.vq_assign(x, 4, cb)
    dec = orc.gather_dequant(orc.Scheme.vq(12, cb), orc.pack(q, 8), np.arange(40))
    assert np.array_equal(dec, x) and dist[-1] == 0


def test_decode_is_codebook_lookup():
    x = _table(200, 20)
    cb, _ = orc.vq_train(x, 5, 16, iters=4)
    q = orc.vq_assign(x, 5, cb)
    dec = orc.gather_dequant(orc.Scheme.vq(20, cb), orc.pack(q, 8), np.arange(200))
    want = np.concatenate([cb[p][q[:, p]] for p in range(4)], axis=1)
    assert np.array_equal(dec, want)


def test_two_well_separated_modes_in_1d():
    rng = np.random.default_rng(2)
    a = rng.normal(0, 0.1, 500)
    b = rng.normal(10, 0.1, 500)
    x = rng.permutation(np.concatenate([a, b])).astype(np.float32)[:, None]
    cb, _ = orc.vq_train(x, 1, 2, iters=10)
    got = np.sort(cb[0, :, 0])
    assert np.allclose(got, [x[x < 5].mean(), x[x > 5].mean()], atol=1e-5)


def test_against_library_kmeans_from_same_start():
    from sklearn.cluster import KMeans
    x = _table(1200, 8)
    length = 8
    cb, dist = orc.vq_train(x, 8, length, iters=10)
    init = np.unique(x, axis=0, return_index=True)[1]
    init = x[np.sort(init)[:length]]                         # first `length` distinct rows
    km = KMeans(n_clusters=length, init=init, n_init=1, max_iter=10, tol=0.0,
                algorithm="lloyd").fit(x.astype(np.float64))
    # sklearn counts the update after its last assignment; compare inertia of
    # the oracle's final codebook with the library's final centres
    def inertia(c):
        return ((x[:, None, :].astype(np.float64) - c[None]) ** 2).sum(-1).min(1).mean()
    assert abs(inertia(cb[0]) - inertia(km.cluster_centers_)) <= 0.02 * inertia(km.cluster_centers_)
