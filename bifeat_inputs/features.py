"""Counter-based node-feature generator (host side, numpy).

Recipe for element (i, j) of an N x D table with a given seed:

    h   = mix64(key_feat + (i*D + j))              64-bit integer mixer
    S   = sum of the four 16-bit lanes of h        integer in [0, 262140]
    z   = float32(S - 131070) * C_Z                one fp32 multiply
    x   = float32(sigma_j * z) + mu_j              fp32 multiply, then fp32 add
    (fp16 tables: x is then rounded to fp16, round-to-nearest-even)

``z`` is a centred 4-term Irwin-Hall variate scaled to unit variance, a
bounded (|z| < 3.47) stand-in for a standard normal; every step is an exactly
specified integer or single correctly-rounded fp32 operation, so host and
device produce the same bits.  Column location/scale are

    mu_j    = 2*u - 1,          u  = top 24 bits of mix64(key_mu + j) * 2^-24
    sigma_j = 1.5*u' + 0.5,     u' = top 24 bits of mix64(key_sigma + j) * 2^-24

computed here once and handed to the device generator as arrays.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# 1 / sqrt(4 * (65536**2 - 1) / 12): unit variance for the sum of four
# independent uniform 16-bit lanes.
C_Z = np.float32(1.0 / np.sqrt(4.0 * (65536.0 ** 2 - 1.0) / 12.0))
S_CENTRE = 131070  # 4 * 65535 / 2

STREAM_FEAT, STREAM_MU, STREAM_SIGMA = 1, 2, 3
STREAM_GRAPH_DEG, STREAM_GRAPH_NBR, STREAM_SEEDS, STREAM_SLOTS = 4, 5, 6, 7
STREAM_MISC = 8


def mix64(z) -> np.ndarray:
    """Finalising 64-bit mixer (two xor-shift-multiply rounds and a last
    xor-shift); wraps modulo 2^64."""
    z = np.asarray(z, dtype=np.uint64).copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def stream_key(seed: int, stream: int) -> np.uint64:
    """Per-(seed, stream) 64-bit key; element counters are added to it."""
    base = (int(seed) * int(_GOLDEN) + int(stream)) & 0xFFFFFFFFFFFFFFFF
    return mix64(np.array([base], dtype=np.uint64))[0]


def _uniform24(key: np.uint64, idx: np.ndarray) -> np.ndarray:
    h = mix64(np.uint64(key) + idx.astype(np.uint64))
    return (h >> np.uint64(40)).astype(np.float32) * np.float32(2.0 ** -24)


def column_params(seed: int, D: int):
    """(mu[D], sigma[D]) fp32: mu ~ U(-1, 1), sigma ~ U(0.5, 2)."""
    j = np.arange(D, dtype=np.uint64)
    u = _uniform24(stream_key(seed, STREAM_MU), j)
    v = _uniform24(stream_key(seed, STREAM_SIGMA), j)
    mu = np.float32(2.0) * u - np.float32(1.0)
    sigma = np.float32(1.5) * v + np.float32(0.5)
    return mu.astype(np.float32), sigma.astype(np.float32)


@dataclass(frozen=True)
class FeatureSpec:
    """A synthetic table: N rows, D columns, seed, storage dtype."""
    N: int
    D: int
    seed: int = 0
    dtype: str = "f32"  # "f32" | "f16"

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float16


def _rows_block(spec: FeatureSpec, rows: np.ndarray, mu, sigma) -> np.ndarray:
    D = spec.D
    e = rows.astype(np.uint64)[:, None] * np.uint64(D) + np.arange(D, dtype=np.uint64)[None, :]
    h = mix64(stream_key(spec.seed, STREAM_FEAT) + e)
    m16 = np.uint64(0xFFFF)
    S = ((h & m16) + ((h >> np.uint64(16)) & m16) + ((h >> np.uint64(32)) & m16)
         + (h >> np.uint64(48))).astype(np.int64)
    z = (S - S_CENTRE).astype(np.float32) * C_Z
    x = sigma[None, :] * z          # fp32 multiply
    x = x + mu[None, :]             # fp32 add
    if spec.dtype == "f16":
        x = x.astype(np.float16)
    return x


def feature_rows(spec: FeatureSpec, rows) -> np.ndarray:
    """Rows ``rows`` (any order, repeats allowed) of the table, [len(rows), D]
    in the table's storage dtype."""
    rows = np.asarray(rows, dtype=np.int64)
    mu, sigma = column_params(spec.seed, spec.D)
    out = np.empty((rows.shape[0], spec.D), dtype=spec.np_dtype)
    step = max(1, (1 << 22) // max(1, spec.D))
    for s in range(0, rows.shape[0], step):
        out[s:s + step] = _rows_block(spec, rows[s:s + step], mu, sigma)
    return out


def feature_chunk(spec: FeatureSpec, row0: int, nrows: int) -> np.ndarray:
    """Rows [row0, row0 + nrows) of the table."""
    return feature_rows(spec, np.arange(row0, row0 + nrows, dtype=np.int64))
