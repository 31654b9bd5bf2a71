"""Pins for the oracle's logarithmic scalar codes (Sec. 3.1, Eq. (1)/(2))."""
import os

import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "log_k3_hand.txt")


def _table(rows=3000, D=16, seed=5):
    return feature_chunk(FeatureSpec(rows, D, seed), 0, rows)


def test_hand_evaluated_example():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    x = np.array([float(r[0]) for r in rows], np.float32)
    want_q = np.array([int(r[1]) for r in rows], np.uint8)
    want_v = np.array([float(r[2]) for r in rows])
    T, V = orc.log_tables(0.0, 4.0, 3)
    assert np.array_equal(T, np.array([2, 4, 8], np.float32))
    q = orc.log_encode(x, 3, T)
    assert np.array_equal(q, want_q)
    assert np.array_equal(orc.log_encode_direct(x, 3, 0.0, 4.0), want_q)
    assert np.allclose(V[q], want_v, rtol=1e-7)     # 3-bit codes have no packed layout


@pytest.mark.parametrize("k", [1, 2, 3, 4, 8])
def test_threshold_form_equals_printed_form(k):
    x = _table()
    e_min, e_max = orc.log_range(orc.log_fit(x))
    T, _ = orc.log_tables(e_min, e_max, k)
    a = orc.log_encode(x, k, T)
    b = orc.log_encode_direct(x, k, e_min, e_max)
    # they may differ only for magnitudes within rounding of a bin edge
    assert (a != b).sum() <= 2
    assert np.abs(a.astype(int) - b.astype(int)).max() <= 1


def test_fit_range_is_log2_of_extreme_magnitudes():
    x = _table().copy()
    x[0, 0] = 0.0
    x[1, 1] = np.nan
    x[2, 2] = np.inf
    st = orc.log_fit(x[:1000])
    st = orc.log_fit(x[1000:], st)
    m = np.abs(x[np.isfinite(x)])
    assert st[0] == m[m > 0].min() and st[1] == m.max()
    e_min, e_max = orc.log_range(st)
    assert np.isclose(e_min, np.log2(float(st[0]))) and np.isclose(e_max, np.log2(float(st[1])))
    assert orc.log_range(np.array([np.inf, 0], np.float32)) == (0.0, 0.0)   # all-zero table


@pytest.mark.parametrize("k", [2, 4, 8])
def test_monotone_symmetric_and_decode_inside_bin(k):
    x = np.sort(_table().reshape(-1))
    e_min, e_max = orc.log_range_clipped(x, 0.01)
    T, V = orc.log_tables(e_min, e_max, k)
    q = orc.log_encode(x, k, T).astype(int)
    assert np.all(np.diff(q) >= 0)                                  # x <= y  =>  Q(x) <= Q(y)
    nz = x != 0
    assert np.array_equal(orc.log_encode(-x[nz], k, T).astype(int), (1 << k) - 1 - q[nz])
    H = 1 << (k - 1)
    edges = np.concatenate([[2.0 ** e_min], T.astype(np.float64), [2.0 ** e_max]])
    for l in range(H):
        assert edges[l] * (1 - 1e-6) <= V[H + l] <= edges[l + 1] * (1 + 1e-6)
        assert V[H - 1 - l] == -V[H + l]
    assert np.all(np.diff(V) > 0)
    # unclipped magnitudes: relative error at most half a bin in log2
    s = orc.Scheme.log(1, V, k)
    dec = orc.gather_dequant(s, orc.pack(q[:, None].astype(np.uint8), k), np.arange(len(x)))[:, 0]
    inside = (np.abs(x) >= 2.0 ** e_min) & (np.abs(x) <= 2.0 ** e_max)
    rel = np.abs(dec[inside].astype(np.float64) / x[inside] - 1)
    half_bin = 2.0 ** ((e_max - e_min) / (2 * H))
    assert rel.max() <= half_bin - 1 + 1e-5
    assert np.all(np.sign(dec[inside]) == np.sign(x[inside]))
    # clipped magnitudes take the extreme levels of their side
    big = np.abs(x) > 2.0 ** e_max
    assert np.all((q[big] == (1 << k) - 1) | (q[big] == 0))
    small = (np.abs(x) < 2.0 ** e_min) & (x > 0)
    assert np.all(q[small] == H)


def test_one_bit_is_the_sign_and_decodes_to_geometric_mean():
    x = _table()
    st = orc.log_fit(x)
    e_min, e_max = orc.log_range(st)
    T, V = orc.log_tables(e_min, e_max, 1)
    assert len(T) == 0
    q = orc.log_encode(x, 1, T)
    assert np.array_equal(q.astype(bool), x > 0)          # "positive or not"; zero with negatives
    gm = np.sqrt(float(st[0]) * float(st[1]))              # exp2((e_min+e_max)/2)
    assert np.isclose(V[1], gm, rtol=1e-6) and V[0] == -V[1]


@pytest.mark.parametrize("k", [1, 2, 4])
def test_binary_features_keep_two_distinct_values(k):
    rng = np.random.default_rng(1)
    x = (rng.random((200, 9)) < 0.4).astype(np.float32)
    e_min, e_max = orc.log_range(orc.log_fit(x))
    assert e_min == 0.0 and e_max == 0.0
    T, V = orc.log_tables(e_min, e_max, k)
    q = orc.log_encode(x, k, T)
    dec = orc.gather_dequant(orc.Scheme.log(9, V, k), orc.pack(q, k), np.arange(200))
    assert np.all(dec[x == 1] == 1.0) and np.all(dec[x == 0] == -1.0)


def test_error_shrinks_with_bits():
    # delta ~ Theta(2^(-32/CR)): more bits, smaller error (Appendix A.5)
    x = _table()
    e_min, e_max = orc.log_range_clipped(x, 0.02)
    errs = []
    for k in [1, 2, 4, 8]:
        T, V = orc.log_tables(e_min, e_max, k)
        q = orc.log_encode(x, k, T)
        dec = orc.gather_dequant(orc.Scheme.log(x.shape[1], V, k), orc.pack(q, k),
                                 np.arange(x.shape[0]))
        errs.append(np.sqrt(((dec - x) ** 2).mean()))
    assert all(a > b for a, b in zip(errs, errs[1:]))


# ---- the clipped range (Sec. 3.1: the range is taken after outliers are clipped; Appendix C
# leaves the fraction open).  The reading: with n finite nonzero magnitudes and fraction p, the
# order statistics at ranks floor(p(n-1)) and ceil((1-p)(n-1)).  Pinned by what an order
# statistic is (a counting property that no sort is needed to state), by numpy's selection
# routine, and by hand-countable cases.
def _count_pin(m, p, e_min, e_max):
    """#{m < v} <= rank < #{m <= v} for both ends, v recovered from the log2 the oracle returns."""
    n = m.size
    lo, hi = np.float32(2.0 ** e_min), np.float32(2.0 ** e_max)
    # the ends are table magnitudes, reproduced exactly by exp2 of their fp64 log2
    assert np.any(m == lo) and np.any(m == hi)
    k_lo = int(np.floor(p * (n - 1)))
    k_hi = int(np.ceil((1.0 - p) * (n - 1)))
    assert (m < lo).sum() <= k_lo < (m <= lo).sum()
    assert (m < hi).sum() <= k_hi < (m <= hi).sum()
    return k_lo, k_hi


@pytest.mark.parametrize("p", [0.0, 0.001, 0.01, 0.05, 0.25, 0.499])
@pytest.mark.parametrize("n", [1, 2, 3, 10, 101, 1000, 4097])
def test_clipped_range_is_the_order_statistic_by_counting(n, p):
    rng = np.random.default_rng(1000 * n + int(1e4 * p))
    x = (rng.standard_normal(n) * np.exp(rng.standard_normal(n))).astype(np.float32)
    x[x == 0] = 1.0
    e_min, e_max = orc.log_range_clipped(x, p)
    m = np.abs(x)
    k_lo, k_hi = _count_pin(m, p, e_min, e_max)
    # a library selection routine on the same ranks
    assert np.float32(2.0 ** e_min) == np.partition(m, k_lo)[k_lo]
    assert np.float32(2.0 ** e_max) == np.partition(m, k_hi)[k_hi]
    assert e_min <= e_max


def test_clipped_range_hand_counted_cases():
    # magnitudes 1, 2, 4, ..., 1024 (n = 11, log2 = 0..10), signs mixed, order shuffled
    x = np.array([-(2.0 ** i) if i % 2 else 2.0 ** i for i in range(11)], dtype=np.float32)[
        [5, 0, 9, 3, 10, 1, 7, 2, 8, 4, 6]]
    # p(n-1) integral: p = 0.1 -> ranks 1 and 9; p = 0.2 -> 2 and 8; p = 0.3 -> 3 and 7
    assert orc.log_range_clipped(x, 0.1) == (1.0, 9.0)
    assert orc.log_range_clipped(x, 0.2) == (2.0, 8.0)
    assert orc.log_range_clipped(x, 0.3) == (3.0, 7.0)
    # fractional ranks: the low end rounds down, the high end up (never clips more than asked)
    assert orc.log_range_clipped(x, 0.15) == (1.0, 9.0)        # 1.5 -> 1,  8.5 -> 9
    assert orc.log_range_clipped(x, 0.25) == (2.0, 8.0)        # 2.5 -> 2,  7.5 -> 8
    assert orc.log_range_clipped(x, 0.05) == (0.0, 10.0)       # 0.5 -> 0,  9.5 -> 10
    assert orc.log_range_clipped(x, 0.0) == (0.0, 10.0)        # no clipping: the extremes
    # both tails are clipped, and symmetrically in rank
    for p in [0.1, 0.2, 0.3, 0.4]:
        e_min, e_max = orc.log_range_clipped(x, p)
        assert e_min == 10.0 - e_max
    # a single value, and all values equal
    assert orc.log_range_clipped(np.array([-8.0], np.float32), 0.3) == (3.0, 3.0)
    assert orc.log_range_clipped(np.full(7, 0.25, np.float32), 0.2) == (-2.0, -2.0)


def test_clipped_range_ignores_zeros_and_non_finite_and_handles_ties():
    # ties: magnitudes 1 x5, 2 x5, 4 x5 -> n = 15; p = 0.2 -> ranks floor(2.8) = 2, ceil(11.2) = 12
    x = np.array([1, -1, 1, -1, 1, 2, -2, 2, -2, 2, 4, -4, 4, -4, 4], dtype=np.float32)
    assert orc.log_range_clipped(x, 0.2) == (0.0, 2.0)
    # p = 0.4 -> ranks floor(5.6) = 5, ceil(8.4) = 9: both inside the run of 2s
    assert orc.log_range_clipped(x, 0.4) == (1.0, 1.0)
    # zeros, NaN and infinities do not count towards n
    y = np.concatenate([x, np.array([0, 0, -0.0, np.nan, np.inf, -np.inf], np.float32)])
    for p in [0.0, 0.2, 0.4]:
        assert orc.log_range_clipped(y, p) == orc.log_range_clipped(x, p)
    assert orc.log_range_clipped(np.array([0, np.nan, np.inf], np.float32), 0.1) == (0.0, 0.0)
    # p = 0 equals the plain fit of the extremes
    t = _table()
    assert orc.log_range_clipped(t, 0.0) == orc.log_range(orc.log_fit(t))
    _count_pin(np.abs(t.reshape(-1))[np.abs(t.reshape(-1)) > 0], 0.01, *orc.log_range_clipped(t, 0.01))
