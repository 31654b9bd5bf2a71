"""Pins for the oracle's uniform scalar quantizer, packing and fit.

Each check is something the mathematics fixes independently of the oracle's
own code: a library routine (numpy min/max, packbits), a brute-force search
over all levels in fp64, the half-step error bound, exact special cases.
"""
import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk


def _table(rows=2000, D=37, seed=3):
    return feature_chunk(FeatureSpec(rows, D, seed), 0, rows)


def test_row_bytes_layout():
    # ceil(D*b/8) rounded up to 16
    assert orc.row_bytes(100, 4) == 64
    assert orc.row_bytes(128, 2) == 32
    assert orc.row_bytes(768, 1) == 96
    assert orc.row_bytes(768, 4) == 384
    assert orc.row_bytes(128, 8) == 128
    assert orc.row_bytes(1, 1) == 16
    # compression ratio 32 for 1 bit per fp32 value (Sec. 3.1): unpadded bytes
    assert (768 * 4) / (768 * 1 / 8) == 32


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_pack_matches_packbits(bits):
    rng = np.random.default_rng(bits)
    D = 53
    q = rng.integers(0, 1 << bits, size=(17, D), dtype=np.uint8)
    packed = orc.pack(q, bits)
    # independent construction: expand each code into its bits LSB-first,
    # concatenate along the row, pack little-endian
    bitplane = ((q[:, :, None] >> np.arange(bits)[None, None, :]) & 1).astype(np.uint8)
    want = np.packbits(bitplane.reshape(17, D * bits), axis=1, bitorder="little")
    assert packed.shape[1] % 16 == 0
    assert np.array_equal(packed[:, :want.shape[1]], want)
    assert not packed[:, want.shape[1]:].any()          # zero padding
    assert np.array_equal(orc.unpack(packed, D, bits), q)


def test_fit_is_min_max():
    x = _table()
    mn, mx = orc.fit_minmax(x[:700])
    mn, mx = orc.fit_minmax(x[700:], mn, mx)             # running update
    assert np.array_equal(mn, x.min(axis=0))
    assert np.array_equal(mx, x.max(axis=0))


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_nearest_level_bruteforce_and_half_step_bound(bits):
    x = _table()
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, bits)
    q = orc.uniform_encode(x, bits, mn, inv)
    L = (1 << bits) - 1
    assert q.max() <= L
    # brute force in fp64 over every level
    levels = mn.astype(np.float64)[None, :] + np.arange(L + 1)[:, None] * \
        ((mx.astype(np.float64) - mn.astype(np.float64)) / L)[None, :]            # [L+1, D]
    dist = np.abs(x.astype(np.float64)[None, :, :] - levels[:, None, :])          # [L+1, rows, D]
    best = dist.min(axis=0)
    mine = np.take_along_axis(dist, q[None].astype(np.int64), axis=0)[0]
    step = (mx.astype(np.float64) - mn.astype(np.float64)) / L
    assert np.all(mine <= best + 1e-6 * step[None, :])
    assert (q == dist.argmin(axis=0)).mean() > 0.9999
    # the decoded value (through pack -> gather -> decode) is within half a step
    s = orc.Scheme.uniform(mn, scale, bits)
    xd = orc.gather_dequant(s, orc.pack(q, bits), np.arange(x.shape[0]))
    ulp = np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)
    bound = scale.astype(np.float64)[None, :] / 2 * (1 + 2.0 ** -20) + ulp
    assert np.all(np.abs(xd.astype(np.float64) - x.astype(np.float64)) <= bound)
    # both extreme codes are used (min -> 0, max -> L)
    assert np.array_equal(q.min(axis=0), np.zeros(x.shape[1], np.uint8))
    assert np.array_equal(q.max(axis=0), np.full(x.shape[1], L, np.uint8))


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_requantizing_grid_points_is_identity(bits):
    x = _table(500, 19)
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, bits)
    L = (1 << bits) - 1
    q = np.tile(np.arange(L + 1, dtype=np.uint8)[:, None], (1, x.shape[1]))
    s = orc.Scheme.uniform(mn, scale, bits)
    grid = orc.gather_dequant(s, orc.pack(q, bits), np.arange(L + 1))
    assert np.array_equal(orc.uniform_encode(grid, bits, mn, inv), q)


def test_constant_column_exact():
    x = _table(300, 8).copy()
    x[:, 3] = np.float32(-0.731)
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, 4)
    assert scale[3] == 0 and inv[3] == 0
    q = orc.uniform_encode(x, 4, mn, inv)
    assert not q[:, 3].any()
    xd = orc.gather_dequant(orc.Scheme.uniform(mn, scale, 4), orc.pack(q, 4), np.arange(300))
    assert np.all(xd[:, 3] == np.float32(-0.731))


def test_one_bit_is_nearer_to_max():
    x = _table()
    mn, mx = orc.fit_minmax(x)
    _, inv = orc.uniform_params(mn, mx, 1)
    q = orc.uniform_encode(x, 1, mn, inv)
    xd = x.astype(np.float64)
    nearer_max = (mx[None, :] - xd) < (xd - mn[None, :])
    tie = np.isclose(mx[None, :] - xd, xd - mn[None, :], rtol=1e-6)
    assert np.array_equal(q[~tie].astype(bool), nearer_max[~tie])


def test_binary_features_are_lossless():
    # Sec. 3.1: one-hot / binary features lose nothing at one bit
    rng = np.random.default_rng(0)
    x = (rng.random((400, 21)) < 0.3).astype(np.float32)
    x[0, :] = 0
    x[1, :] = 1
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, 1)
    q = orc.uniform_encode(x, 1, mn, inv)
    assert np.array_equal(q, x.astype(np.uint8))
    xd = orc.gather_dequant(orc.Scheme.uniform(mn, scale, 1), orc.pack(q, 1), np.arange(400))
    assert np.array_equal(xd, x)


def test_ties_round_to_even_and_clamp_and_nan():
    L = 15
    mn = np.zeros(1, np.float32)
    mx = np.full(1, L, np.float32)                  # step exactly 1
    scale, inv = orc.uniform_params(mn, mx, 4)
    assert scale[0] == 1 and inv[0] == 1
    x = np.array([[0.5], [1.5], [2.5], [3.5], [-7.0], [99.0], [np.nan], [14.5]], np.float32)
    q = orc.uniform_encode(x, 4, mn, inv)[:, 0]
    assert list(q) == [0, 2, 2, 4, 0, 15, 0, 14]


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_rms_error_is_step_over_sqrt12(bits):
    # smooth density, step small against the spread: error ~ U(-step/2, step/2)
    x = _table(20000, 6)
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, bits)
    q = orc.uniform_encode(x, bits, mn, inv)
    xd = orc.gather_dequant(orc.Scheme.uniform(mn, scale, bits), orc.pack(q, bits),
                            np.arange(x.shape[0]))
    rms = np.sqrt(((xd.astype(np.float64) - x) ** 2).mean(axis=0))
    tol = {2: 0.25, 4: 0.05, 8: 0.03}[bits]
    assert np.allclose(rms, scale / np.sqrt(12), rtol=tol)
