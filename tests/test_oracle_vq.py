"""Pins for the oracle's vector codes (Sec. 3.2, Appendix C)."""
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


# ------------------------------------------------- the variants of Sec. 3.2 / Appendix C
def _margin_filter(score, q, rtol):
    """Rows whose best and second-best scores are clearly apart."""
    part = np.partition(score, -2, axis=1)
    return (part[:, -1] - part[:, -2]) > rtol * np.abs(part[:, -1])


@pytest.mark.parametrize("w,length", [(8, 64), (5, 7), (16, 300)])
def test_cosine_assign_is_bruteforce_most_similar(w, length):
    x = _table(800, 40)
    D = x.shape[1]
    P = orc.vq_parts(D, w)
    cb = np.random.default_rng(3 * w).normal(size=(P, length, w)).astype(np.float32)
    q = orc.vq_assign(x, w, cb, metric="cosine")
    assert q.dtype == (np.uint16 if length > 256 else np.uint8)
    xp = np.zeros((x.shape[0], P * w))
    xp[:, :D] = x
    for p in range(P):
        sub = xp[:, p * w:(p + 1) * w]
        c = cb[p].astype(np.float64)
        cos = (sub @ c.T) / np.linalg.norm(c, axis=1)[None, :] / np.linalg.norm(sub, axis=1)[:, None]
        clear = _margin_filter(cos, q, 1e-5)
        assert clear.mean() > 0.99
        assert np.array_equal(cos.argmax(1)[clear], q[clear, p])


def test_cosine_ignores_positive_scaling_and_l2_does_not():
    x = _table(500, 16)
    cb = np.random.default_rng(5).normal(size=(2, 32, 8)).astype(np.float32)
    q1 = orc.vq_assign(x, 8, cb, metric="cosine")
    # powers of two scale every product exactly, so the argmax cannot move
    assert np.array_equal(q1, orc.vq_assign(4.0 * x, 8, cb, metric="cosine"))
    assert np.array_equal(q1, orc.vq_assign(x, 8, 0.5 * cb, metric="cosine"))
    # entry norms matter to the Euclidean search but not to the cosine one
    scaled = cb * np.linspace(0.2, 5, 32, dtype=np.float32)[None, :, None]
    agree = orc.vq_assign(x, 8, scaled, metric="cosine") == q1
    assert agree.mean() > 0.99           # entry norms change only rounding-level ties
    assert (orc.vq_assign(x, 8, scaled) != orc.vq_assign(x, 8, cb)).mean() > 0.2


def test_cosine_equals_euclidean_on_the_unit_sphere():
    # |x - c|^2 = 2 - 2 cos for unit vectors: both searches pick the same entry
    rng = np.random.default_rng(9)
    x = rng.normal(size=(600, 8))
    x = (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)
    c = rng.normal(size=(1, 50, 8))
    c = (c / np.linalg.norm(c, axis=2, keepdims=True)).astype(np.float32)
    a, b = orc.vq_assign(x, 8, c, metric="cosine")[:, 0], orc.vq_assign(x, 8, c)[:, 0]
    cos = x.astype(np.float64) @ c[0].astype(np.float64).T
    clear = _margin_filter(cos, a, 1e-5)
    assert clear.mean() > 0.98 and np.array_equal(a[clear], b[clear])


def test_cosine_degenerate_parts():
    cb = np.zeros((1, 3, 2), np.float32)
    cb[0, 1] = [1, 0]
    cb[0, 2] = [-1, 0]
    x = np.array([[0, 0], [2, 0], [-3, 0], [0, 5]], np.float32)
    # zero row: every score 0 -> entry 0; orthogonal row: all scores 0 -> entry 0 (an
    # all-zero entry scores 0 as well)
    assert list(orc.vq_assign(x, 2, cb, metric="cosine")[:, 0]) == [0, 1, 2, 0]
    assert np.array_equal(orc.vq_rnorm(cb)[0], np.array([0, 1, 1], np.float32))


def test_rnorm_is_the_rounded_reciprocal_norm():
    cb = np.random.default_rng(2).normal(size=(3, 40, 6)).astype(np.float32)
    want = (1.0 / np.sqrt((cb.astype(np.float64) ** 2).sum(-1))).astype(np.float32)
    got = orc.vq_rnorm(cb)
    # same value up to the summation order inside numpy's reduction (1 ulp)
    assert np.allclose(got, want, rtol=1.2e-7, atol=0)


def test_two_byte_codes_layout_and_roundtrip():
    q = np.array([[0x0102, 0x3FFF, 7], [300, 0, 0x1234]], dtype=np.uint16)
    packed = orc.pack(q, 16)
    assert packed.shape == (2, 16) and orc.row_bytes(3, 16) == 16
    assert list(packed[0, :6]) == [0x02, 0x01, 0xFF, 0x3F, 7, 0] and not packed[:, 6:].any()
    assert np.array_equal(orc.unpack(packed, 3, 16), q)
    big = np.random.default_rng(0).integers(0, 16384, (37, 11)).astype(np.uint16)
    assert orc.pack(big, 16).shape == (37, 32)
    assert np.array_equal(orc.unpack(orc.pack(big, 16), 11, 16), big)


@pytest.mark.parametrize("metric", ["l2", "cosine"])
def test_large_codebook_assign_and_decode(metric):
    x = _table(400, 20)
    w, length = 4, 1000
    P = orc.vq_parts(20, w)
    cb = np.random.default_rng(11).normal(size=(P, length, w)).astype(np.float32)
    q = orc.vq_assign(x, w, cb, metric=metric)
    assert q.dtype == np.uint16 and q.max() > 255
    if metric == "l2":
        d2 = ((x.reshape(400, P, 1, w).astype(np.float64) - cb.astype(np.float64)[None]) ** 2).sum(-1)
        assert (d2.argmin(2) == q).mean() > 0.995
    s = orc.Scheme.vq(20, cb)
    assert s.row_bytes == 16 and s.bits == 16
    idx = np.array([5, 0, 399, 5])
    dec = orc.gather_dequant(s, orc.pack(q, 16), idx)
    want = cb[np.arange(P)[None, :], q[idx]].reshape(4, P * w)
    assert np.array_equal(dec, want)
    # mean of two rows = average of their decoded rows
    m = orc.gather_mean(s, orc.pack(q, 16), np.array([0, 2, 2]), np.array([5, 0]))
    assert np.allclose(m[0], (want[0].astype(np.float64) + want[1]) / 2, rtol=1e-7) and not m[1].any()


def test_cosine_training_round_is_assign_then_member_means():
    x = _table(700, 16)
    w, length = 8, 12
    cb1, d1 = orc.vq_train(x, w, length, iters=1, metric="cosine")
    cb2, d2 = orc.vq_train(x, w, length, iters=2, metric="cosine")
    assert d1[0] == d2[0]
    # the second round, redone by hand from the first round's codebooks
    q = orc.vq_assign(x, w, cb1, metric="cosine")
    for p in range(2):
        sub = x[:, p * w:(p + 1) * w].astype(np.float64)
        for c in range(length):
            mem = sub[q[:, p] == c]
            want = mem.mean(0).astype(np.float32) if len(mem) else cb1[p, c]
            assert np.allclose(cb2[p, c], want, rtol=1e-6, atol=1e-7)
    dec = cb1[np.arange(2)[None, :], q].reshape(700, 16).astype(np.float64)
    assert np.isclose(d2[1], ((x - dec) ** 2).sum() / 700, rtol=1e-9)


def test_l2_training_via_the_metric_entry_matches_the_plain_one():
    x = _table(600, 16)
    a, da = orc.vq_train(x, 4, 16, iters=4)
    cb = np.zeros_like(a)
    dist = np.zeros(4)
    import ctypes as C
    orc.lib().orc_vq_train_metric(x.ctypes.data_as(C.c_void_p), C.c_int64(600), C.c_int64(16),
                                  C.c_int(4), C.c_int(16), C.c_int(4), C.c_int(0),
                                  cb.ctypes.data_as(C.c_void_p), dist.ctypes.data_as(C.c_void_p))
    assert np.array_equal(a, cb) and np.allclose(da, dist, rtol=1e-5)
