"""CPU oracle for the BiFeat feature-loading path: TEST INFRASTRUCTURE.

Thin ctypes/numpy wrapper over ``bifeat_oracle.c`` (plain C, fp64 decode and
mean, fp32-decided codes).  Only ``tests/``, the smoke check and the
benchmark's CPU-baseline leg import this package; the product never does and
shares no code with it.

``build()`` compiles the C file with gcc; it is also called lazily on first use
when the shared object is missing or older than its source.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bifeat_oracle.c")
_SO = os.path.join(_HERE, "libbifeat_oracle.so")

UNIFORM, LOG, VQ = 0, 1, 2


def build(force: bool = False) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


class _Scheme(C.Structure):
    _fields_ = [("kind", C.c_int32), ("bits", C.c_int32), ("D", C.c_int64),
                ("w", C.c_int32), ("len", C.c_int32),
                ("a", C.c_void_p), ("b", C.c_void_p), ("cb", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_row_bytes.restype = C.c_int64
        _lib.orc_row_bytes.argtypes = [C.c_int64, C.c_int]
        _lib.orc_scheme_row_bytes.restype = C.c_int64
        _lib.orc_max_threads.restype = C.c_int
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def set_threads(n: int) -> None:
    lib().orc_set_threads(C.c_int(n))


def max_threads() -> int:
    return int(lib().orc_max_threads())


# ---------------------------------------------------------------- packing
def row_bytes(ncodes: int, bits: int) -> int:
    return int(lib().orc_row_bytes(ncodes, bits))


def pack(q: np.ndarray, bits: int) -> np.ndarray:
    if bits == 16:       # two-byte vector codes
        q = np.ascontiguousarray(q, dtype=np.uint16)
        rows, n = q.shape
        out = np.empty((rows, row_bytes(n, 16)), dtype=np.uint8)
        lib().orc_pack16(_p(q), C.c_int64(rows), C.c_int64(n), _p(out))
        return out
    assert bits in (1, 2, 4, 8), "codes never straddle a byte"
    q = _u8(q)
    rows, n = q.shape
    out = np.empty((rows, row_bytes(n, bits)), dtype=np.uint8)
    lib().orc_pack(_p(q), C.c_int64(rows), C.c_int64(n), C.c_int(bits), _p(out))
    return out


def unpack(packed: np.ndarray, ncodes: int, bits: int) -> np.ndarray:
    if bits == 16:
        packed = _u8(packed)
        assert packed.shape[1] == row_bytes(ncodes, 16)
        out = np.empty((packed.shape[0], ncodes), dtype=np.uint16)
        lib().orc_unpack16(_p(packed), C.c_int64(packed.shape[0]), C.c_int64(ncodes), _p(out))
        return out
    assert bits in (1, 2, 4, 8)
    packed = _u8(packed)
    rows = packed.shape[0]
    assert packed.shape[1] == row_bytes(ncodes, bits)
    out = np.empty((rows, ncodes), dtype=np.uint8)
    lib().orc_unpack(_p(packed), C.c_int64(rows), C.c_int64(ncodes), C.c_int(bits), _p(out))
    return out


# ---------------------------------------------------------------- uniform
def fit_minmax(x: np.ndarray, mn: np.ndarray | None = None, mx: np.ndarray | None = None):
    """Running per-column (min, max); pass the previous pair to continue."""
    x = _f32(x)
    rows, D = x.shape
    if mn is None:
        mn = np.full(D, np.inf, dtype=np.float32)
        mx = np.full(D, -np.inf, dtype=np.float32)
    lib().orc_fit_minmax(_p(x), C.c_int64(rows), C.c_int64(D), _p(mn), _p(mx))
    return mn, mx


def uniform_params(mn, mx, bits: int):
    mn, mx = _f32(mn), _f32(mx)
    scale = np.empty_like(mn)
    inv = np.empty_like(mn)
    lib().orc_uniform_params(_p(mn), _p(mx), C.c_int64(mn.shape[0]), C.c_int(bits),
                             _p(scale), _p(inv))
    return scale, inv


def uniform_encode(x, bits: int, mn, inv) -> np.ndarray:
    x, mn, inv = _f32(x), _f32(mn), _f32(inv)
    rows, D = x.shape
    q = np.empty((rows, D), dtype=np.uint8)
    lib().orc_uniform_encode(_p(x), C.c_int64(rows), C.c_int64(D), C.c_int(bits),
                             _p(mn), _p(inv), _p(q))
    return q


# -------------------------------------------------------------------- log
def log_fit(x, state=None):
    """Running (min nonzero |x|, max |x|) as a 2-element fp32 array."""
    x = _f32(x).reshape(-1)
    if state is None:
        state = np.array([np.inf, 0.0], dtype=np.float32)
    lib().orc_log_fit(_p(x), C.c_int64(x.shape[0]), _p(state[0:1]), _p(state[1:2]))
    return state


def log_range(state) -> tuple[float, float]:
    e = np.zeros(2, dtype=np.float64)
    lib().orc_log_range(C.c_float(float(state[0])), C.c_float(float(state[1])),
                        _p(e[0:1]), _p(e[1:2]))
    return float(e[0]), float(e[1])


def log_range_clipped(x, p: float) -> tuple[float, float]:
    """(e_min, e_max) with a fraction p of the nonzero magnitudes clipped at
    each tail (Sec. 3.1 takes the range after outliers are clipped; Appendix C calls the
    fraction a minor setting): the order statistics of |x| at ranks
    floor(p*(n-1)) and ceil((1-p)*(n-1)), by a full sort."""
    m = np.abs(_f32(x).reshape(-1))
    m = np.sort(m[np.isfinite(m) & (m > 0)])
    if m.size == 0:
        return 0.0, 0.0
    lo = m[int(np.floor(p * (m.size - 1)))]
    hi = m[int(np.ceil((1.0 - p) * (m.size - 1)))]
    return log_range(np.array([lo, hi], dtype=np.float32))


def log_tables(e_min: float, e_max: float, k: int):
    H = 1 << (k - 1)
    T = np.zeros(max(H - 1, 1), dtype=np.float32)
    V = np.zeros(1 << k, dtype=np.float32)
    lib().orc_log_tables(C.c_double(e_min), C.c_double(e_max), C.c_int(k), _p(T), _p(V))
    return T[:H - 1].copy(), V


def log_encode(x, k: int, T) -> np.ndarray:
    x = _f32(x)
    T = _f32(T) if len(T) else np.zeros(1, dtype=np.float32)
    q = np.empty(x.shape, dtype=np.uint8)
    lib().orc_log_encode(_p(x), C.c_int64(x.size), C.c_int(k), _p(T), _p(q))
    return q


def log_encode_direct(x, k: int, e_min: float, e_max: float) -> np.ndarray:
    x = _f32(x)
    q = np.empty(x.shape, dtype=np.uint8)
    lib().orc_log_encode_direct(_p(x), C.c_int64(x.size), C.c_int(k), C.c_double(e_min),
                                C.c_double(e_max), _p(q))
    return q


# --------------------------------------------------------------------- vq
def vq_parts(D: int, w: int) -> int:
    return (D + w - 1) // w


METRICS = {"l2": 0, "cosine": 1}


def vq_code_bits(length: int) -> int:
    """Bits per stored index: one byte up to 256 entries, two beyond (Appendix C)."""
    return 8 if length <= 256 else 16


def vq_rnorm(cb) -> np.ndarray:
    """1/|entry| per codebook entry (0 for an all-zero entry), [P, length] fp32."""
    cb = _f32(cb)
    P, length, w = cb.shape
    out = np.empty((P, length), dtype=np.float32)
    lib().orc_vq_rnorm(_p(cb), C.c_int64(P * length), C.c_int(w), _p(out))
    return out


def vq_assign(x, w: int, cb, metric: str = "l2") -> np.ndarray:
    """Indices [rows, P]: uint8 for codebooks of up to 256 entries, else uint16."""
    x, cb = _f32(x), _f32(cb)
    rows, D = x.shape
    P, length, w2 = cb.shape
    assert w2 == w and P == vq_parts(D, w) and 2 <= length <= 16384 and w <= 256
    if metric != "l2" or length > 256:
        q16 = np.empty((rows, P), dtype=np.uint16)
        lib().orc_vq_assign16(_p(x), C.c_int64(rows), C.c_int64(D), C.c_int(w), C.c_int(length),
                              _p(cb), C.c_int(METRICS[metric]), _p(q16))
        return q16 if length > 256 else q16.astype(np.uint8)
    q = np.empty((rows, P), dtype=np.uint8)
    lib().orc_vq_assign(_p(x), C.c_int64(rows), C.c_int64(D), C.c_int(w), C.c_int(length),
                        _p(cb), _p(q))
    return q


def vq_train(sample, w: int, length: int, iters: int = 10, metric: str = "l2"):
    """Returns (codebooks [P, length, w] fp32, distortion per Lloyd round)."""
    sample = _f32(sample)
    ns, D = sample.shape
    cb = np.zeros((vq_parts(D, w), length, w), dtype=np.float32)
    dist = np.zeros(iters, dtype=np.float64)
    if metric != "l2":
        lib().orc_vq_train_metric(_p(sample), C.c_int64(ns), C.c_int64(D), C.c_int(w),
                                  C.c_int(length), C.c_int(iters), C.c_int(METRICS[metric]),
                                  _p(cb), _p(dist))
        return cb, dist
    lib().orc_vq_train(_p(sample), C.c_int64(ns), C.c_int64(D), C.c_int(w), C.c_int(length),
                       C.c_int(iters), _p(cb), _p(dist))
    return cb, dist


# ---------------------------------------------------------------- schemes
class Scheme:
    """Decoder-side description of a packed table (keeps its arrays alive)."""

    def __init__(self, kind: int, D: int, bits: int = 8, a=None, b=None, cb=None):
        self.kind, self.D, self.bits = kind, int(D), int(bits)
        self.a = _f32(a) if a is not None else None
        self.b = _f32(b) if b is not None else None
        self.cb = _f32(cb) if cb is not None else None
        self.w = int(self.cb.shape[2]) if self.cb is not None else 0
        self.len = int(self.cb.shape[1]) if self.cb is not None else 0
        if kind == UNIFORM:
            assert self.a.shape == (D,) and self.b.shape == (D,)
        elif kind == LOG:
            assert self.a.shape == (1 << bits,)
        else:
            assert self.cb.shape[0] == vq_parts(D, self.w) and self.len <= 16384
            self.bits = vq_code_bits(self.len)
        self._c = _Scheme(kind, self.bits, self.D, self.w, self.len,
                          _p(self.a) if self.a is not None else None,
                          _p(self.b) if self.b is not None else None,
                          _p(self.cb) if self.cb is not None else None)

    @classmethod
    def uniform(cls, mn, scale, bits):
        return cls(UNIFORM, len(mn), bits, a=mn, b=scale)

    @classmethod
    def log(cls, D, V, k):
        return cls(LOG, D, k, a=V)

    @classmethod
    def vq(cls, D, cb):
        return cls(VQ, D, 8, cb=cb)

    @property
    def ncodes(self) -> int:
        return vq_parts(self.D, self.w) if self.kind == VQ else self.D

    @property
    def row_bytes(self) -> int:
        return int(lib().orc_scheme_row_bytes(C.byref(self._c)))


def gather_codes(codes, idx) -> np.ndarray:
    codes, idx = _u8(codes), _i64(idx)
    rb = codes.shape[1]
    out = np.empty((idx.shape[0], rb), dtype=np.uint8)
    lib().orc_gather_codes(_p(codes), C.c_int64(rb), _p(idx), C.c_int64(idx.shape[0]), _p(out))
    return out


def gather_dequant(s: Scheme, codes, idx) -> np.ndarray:
    codes, idx = _u8(codes), _i64(idx)
    assert codes.shape[1] == s.row_bytes
    out = np.empty((idx.shape[0], s.D), dtype=np.float32)
    lib().orc_gather_dequant(C.byref(s._c), _p(codes), _p(idx), C.c_int64(idx.shape[0]), _p(out))
    return out


def gather_mean(s: Scheme, codes, indptr, indices) -> np.ndarray:
    codes, indptr, indices = _u8(codes), _i64(indptr), _i64(indices)
    assert codes.shape[1] == s.row_bytes
    V = indptr.shape[0] - 1
    out = np.empty((V, s.D), dtype=np.float32)
    lib().orc_gather_mean(C.byref(s._c), _p(codes), _p(indptr), _p(indices), C.c_int64(V), _p(out))
    return out


def gather_sum(s: Scheme, codes, indptr, indices) -> np.ndarray:
    codes, indptr, indices = _u8(codes), _i64(indptr), _i64(indices)
    assert codes.shape[1] == s.row_bytes
    V = indptr.shape[0] - 1
    out = np.empty((V, s.D), dtype=np.float32)
    lib().orc_gather_sum(C.byref(s._c), _p(codes), _p(indptr), _p(indices), C.c_int64(V), _p(out))
    return out


# ------------------------------------- later layers, aggregation scale factors
def aggregate_rows(x, indptr, indices, sum: bool = False) -> np.ndarray:
    """Appendix A.1 for layers after the first: mean (or sum) of fp32 rows over
    the listed neighbours."""
    x, indptr, indices = _f32(x), _i64(indptr), _i64(indices)
    V = indptr.shape[0] - 1
    out = np.empty((V, x.shape[1]), dtype=np.float32)
    lib().orc_aggregate_rows(_p(x), C.c_int64(x.shape[1]), _p(indptr), _p(indices), C.c_int64(V),
                             C.c_int(1 if sum else 0), _p(out))
    return out


def gather_mean_2hop(s: Scheme, codes, indptr1, indices1, indptr2, indices2) -> np.ndarray:
    """Appendix A.1 applied twice with nothing in between: the mean over the seed
    block's lists of the means over the outer block's lists of decoded rows."""
    codes = _u8(codes)
    indptr1, indices1, indptr2, indices2 = _i64(indptr1), _i64(indices1), _i64(indptr2), _i64(indices2)
    assert codes.shape[1] == s.row_bytes
    V2 = indptr2.shape[0] - 1
    out = np.empty((V2, s.D), dtype=np.float32)
    lib().orc_gather_mean_2hop(C.byref(s._c), _p(codes), _p(indptr1), _p(indices1), _p(indptr2),
                               _p(indices2), C.c_int64(V2), _p(out))
    return out


def scale_profile(x, indptr, indices, layers: int) -> np.ndarray:
    """Appendix A.1 / A.5: mean row length after 0..layers rounds of
    neighbourhood averaging over the whole graph (fp64)."""
    x, indptr, indices = _f32(x), _i64(indptr), _i64(indices)
    n = indptr.shape[0] - 1
    assert x.shape[0] == n
    out = np.empty(layers + 1, dtype=np.float64)
    lib().orc_scale_profile(_p(x), C.c_int64(n), C.c_int64(x.shape[1]), _p(indptr), _p(indices),
                            C.c_int(layers), _p(out))
    return out
