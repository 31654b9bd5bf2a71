"""ctypes binding of the C ABI in ``include/bifeat.h``: same names, argument
marshalling only.  Tensors are torch CUDA tensors; their ``data_ptr()`` and the
current stream's handle are what crosses the boundary."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("BIFEAT_LIB") or os.path.join(_HERE, "libbifeat.so")

UNIFORM, LOG, VQ = 0, 1, 2
VQ_L2, VQ_COSINE = 0, 1
F32, F16 = 0, 1
OK, EINVAL, ENOTFIT, EHIP, ENOTSUP, ELIMIT = 0, -1, -2, -3, -4, -5
FIT_AGAIN = 1


class BifeatError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"bifeat: {text} (status {status})")
        self.status = status


class _CScheme(C.Structure):
    _fields_ = [("kind", C.c_int32), ("bits", C.c_int32),
                ("vq_width", C.c_int32), ("vq_length", C.c_int32), ("vq_metric", C.c_int32)]


@dataclass(frozen=True)
class Scheme:
    kind: int
    bits: int = 8
    vq_width: int = 0
    vq_length: int = 0
    vq_metric: int = 0


_lib = None

_SIGNATURES = {
    "bifeat_params_create": (C.c_int, [C.POINTER(_CScheme), C.c_int64, C.POINTER(C.c_void_p)]),
    "bifeat_params_destroy": (None, [C.c_void_p]),
    "bifeat_row_bytes": (C.c_int64, [C.c_void_p]),
    "bifeat_codes_per_row": (C.c_int64, [C.c_void_p]),
    "bifeat_fit_reset": (C.c_int, [C.c_void_p, C.c_void_p]),
    "bifeat_fit_update": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p]),
    "bifeat_fit_finalize": (C.c_int, [C.c_void_p, C.c_void_p]),
    "bifeat_fit_set_log_clip": (C.c_int, [C.c_void_p, C.c_double]),
    "bifeat_params_set_uniform": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "bifeat_params_get_uniform": (C.c_int, [C.c_void_p] + [C.c_void_p] * 4),
    "bifeat_params_set_log": (C.c_int, [C.c_void_p, C.c_double, C.c_double]),
    "bifeat_params_get_log": (C.c_int, [C.c_void_p] + [C.c_void_p] * 4),
    "bifeat_params_set_codebooks": (C.c_int, [C.c_void_p, C.c_void_p]),
    "bifeat_params_get_codebooks": (C.c_int, [C.c_void_p, C.c_void_p]),
    "bifeat_vq_distortion": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32]),
    "bifeat_produce_fit_begin": (C.c_int, [C.c_void_p, C.c_void_p]),
    "bifeat_produce_fit_end": (C.c_int, [C.c_void_p, C.c_int64]),
    "bifeat_produce_quantize_check": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64]),
    "bifeat_quantize": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p,
                                  C.c_int64, C.c_void_p]),
    "bifeat_gather_codes": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                      C.c_void_p, C.c_void_p]),
    "bifeat_gather_dequant": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                        C.c_void_p, C.c_void_p]),
    "bifeat_gather_dequant_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                               C.c_void_p, C.c_void_p]),
    "bifeat_gather_mean": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "bifeat_gather_sum": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "bifeat_gather_mean_2hop": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64,
                                          C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                          C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                          C.c_void_p, C.c_void_p]),
    "bifeat_gather_mean_i32": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                         C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "bifeat_gather_sum_i32": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                        C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "bifeat_poll_status": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32]),
    "bifeat_reserve": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p]),
    "bifeat_aggregate_rows": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                        C.c_int64, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]),
    "bifeat_check_lists": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p]),
    "bifeat_scale_profile": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                       C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "bifeat_strerror": (C.c_char_p, [C.c_int]),
    "bifeat_set_option": (C.c_int, [C.c_void_p, C.c_char_p, C.c_int]),
}


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libbifeat.so (built by ``paper_2207_14696_amd.build``).  No fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with "
                              "`python -m paper_2207_14696_amd.build`")
        lib = C.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(status: int) -> None:
    if status != OK:
        raise BifeatError(status, load_library().bifeat_strerror(status).decode())


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dev_ptr(t, dtypes=None) -> int:
    if t is None:
        return 0
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    if dtypes is not None and t.dtype not in dtypes:
        raise ValueError(f"unexpected dtype {t.dtype}")
    return t.data_ptr()


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Quantizer:
    """Owns a ``bifeat_params`` handle.  Method names follow the C entry points
    (``bifeat_`` prefix dropped)."""

    def __init__(self, scheme: Scheme, D: int, row_align: int = 16):
        """row_align: option "row_align" of the library (16: rows back to back; 128: rows laid
        out so that none straddles a 128-byte line needlessly), set before anything is packed."""
        self._lib = load_library()
        self.scheme, self.D = scheme, int(D)
        h = C.c_void_p()
        cs = _CScheme(scheme.kind, scheme.bits, scheme.vq_width, scheme.vq_length, scheme.vq_metric)
        _check(self._lib.bifeat_params_create(C.byref(cs), self.D, C.byref(h)))
        self._h = h
        if row_align != 16:
            self.set_option("row_align", row_align)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            self._lib.bifeat_params_destroy(h)

    # ---- sizes
    @property
    def row_bytes(self) -> int:
        return int(self._lib.bifeat_row_bytes(self._h))

    @property
    def codes_per_row(self) -> int:
        return int(self._lib.bifeat_codes_per_row(self._h))

    def set_option(self, name: str, value: int) -> None:
        _check(self._lib.bifeat_set_option(self._h, name.encode(), int(value)))

    # ---- fit
    @staticmethod
    def _dtype(t) -> int:
        import torch
        if t.dtype == torch.float32:
            return F32
        if t.dtype == torch.float16:
            return F16
        raise ValueError("chunk must be float32 or float16")

    def fit_reset(self) -> None:
        _check(self._lib.bifeat_fit_reset(self._h, _stream()))

    def fit_update(self, chunk) -> None:
        rows = chunk.shape[0]
        _check(self._lib.bifeat_fit_update(self._h, _dev_ptr(chunk), self._dtype(chunk), rows,
                                           _stream()))

    def fit_set_log_clip(self, fraction: float) -> None:
        _check(self._lib.bifeat_fit_set_log_clip(self._h, float(fraction)))

    def fit_finalize(self) -> bool:
        """True when the fit needs another pass over the same chunks (clipped
        logarithmic range: three passes), False when the parameters are ready."""
        status = self._lib.bifeat_fit_finalize(self._h, _stream())
        if status == FIT_AGAIN:
            return True
        _check(status)
        return False

    # ---- parameters (host numpy arrays)
    def params_set_uniform(self, mn, mx) -> None:
        mn = np.ascontiguousarray(mn, np.float32)
        mx = np.ascontiguousarray(mx, np.float32)
        assert mn.shape == (self.D,) and mx.shape == (self.D,)
        _check(self._lib.bifeat_params_set_uniform(self._h, _np_ptr(mn), _np_ptr(mx)))

    def params_get_uniform(self):
        out = [np.empty(self.D, np.float32) for _ in range(4)]
        _check(self._lib.bifeat_params_get_uniform(self._h, *[_np_ptr(a) for a in out]))
        return tuple(out)  # min, max, scale, inv

    def params_set_log(self, e_min: float, e_max: float) -> None:
        _check(self._lib.bifeat_params_set_log(self._h, float(e_min), float(e_max)))

    def params_get_log(self):
        k = self.scheme.bits
        e = np.zeros(2, np.float64)
        T = np.zeros(max((1 << (k - 1)) - 1, 1), np.float32)
        V = np.zeros(1 << k, np.float32)
        _check(self._lib.bifeat_params_get_log(self._h, _np_ptr(e[0:1]), _np_ptr(e[1:2]),
                                               _np_ptr(T), _np_ptr(V)))
        return float(e[0]), float(e[1]), T[:(1 << (k - 1)) - 1].copy(), V

    def params_set_codebooks(self, cb) -> None:
        cb = np.ascontiguousarray(cb, np.float32)
        assert cb.shape == (self.codes_per_row, self.scheme.vq_length, self.scheme.vq_width)
        _check(self._lib.bifeat_params_set_codebooks(self._h, _np_ptr(cb)))

    def params_get_codebooks(self):
        cb = np.empty((self.codes_per_row, self.scheme.vq_length, self.scheme.vq_width), np.float32)
        _check(self._lib.bifeat_params_get_codebooks(self._h, _np_ptr(cb)))
        return cb

    def vq_distortion(self, n: int = 10):
        out = np.zeros(n, np.float32)
        _check(self._lib.bifeat_vq_distortion(self._h, _np_ptr(out), n))
        return out

    # ---- encode
    def quantize(self, chunk, codes, row0: int) -> None:
        """codes: uint8 CUDA tensor [N, row_bytes]; rows [row0, row0+len(chunk)) are written."""
        import torch
        rows = chunk.shape[0]
        if codes.dtype != torch.uint8 or codes.shape[1] != self.row_bytes \
                or row0 < 0 or row0 + rows > codes.shape[0] or chunk.shape[1] != self.D:
            raise ValueError("shape mismatch")
        _check(self._lib.bifeat_quantize(self._h, _dev_ptr(chunk), self._dtype(chunk), rows,
                                         _dev_ptr(codes), row0, _stream()))

    # ---- per-iteration load
    def gather_codes(self, codes, idx, out=None):
        import torch
        M = idx.shape[0]
        if out is None:
            out = torch.empty((M, self.row_bytes), dtype=torch.uint8, device=codes.device)
        _check(self._lib.bifeat_gather_codes(self._h, _dev_ptr(codes, (torch.uint8,)),
                                             codes.shape[0], _dev_ptr(idx, (torch.int64,)), M,
                                             _dev_ptr(out, (torch.uint8,)), _stream()))
        return out

    def gather_dequant(self, codes, idx, out=None):
        import torch
        M = idx.shape[0]
        if out is None:
            out = torch.empty((M, self.D), dtype=torch.float32, device=codes.device)
        elif out.shape != (M, self.D):
            raise ValueError("out must be [M, D]")
        _check(self._lib.bifeat_gather_dequant(self._h, _dev_ptr(codes, (torch.uint8,)),
                                               codes.shape[0], _dev_ptr(idx, (torch.int64,)), M,
                                               _dev_ptr(out, (torch.float32,)), _stream()))
        return out

    def gather_dequant_static(self, codes, idx, out):
        """``bifeat_gather_dequant_static``: as gather_dequant, allocating nothing (``out`` is
        required; the workspace is the library's fixed per-GPU array)."""
        import torch
        M = idx.shape[0]
        if out.shape != (M, self.D):
            raise ValueError("out must be [M, D]")
        _check(self._lib.bifeat_gather_dequant_static(
            self._h, _dev_ptr(codes, (torch.uint8,)), codes.shape[0], _dev_ptr(idx, (torch.int64,)), M,
            _dev_ptr(out, (torch.float32,)), _stream()))
        return out

    def _aggregate(self, fn64, fn32, codes, indptr, indices, out):
        import torch
        V = indptr.shape[0] - 1
        if out is None:
            out = torch.empty((V, self.D), dtype=torch.float32, device=codes.device)
        elif out.shape != (V, self.D):
            raise ValueError("out must be [V, D]")
        # int32 list entries go to the _i32 entry point, int64 ones to the plain one
        fn = fn32 if indices.dtype == torch.int32 else fn64
        _check(fn(self._h, _dev_ptr(codes, (torch.uint8,)), codes.shape[0],
                  _dev_ptr(indptr, (torch.int64,)), _dev_ptr(indices, (torch.int64, torch.int32)), V,
                  indices.shape[0], _dev_ptr(out, (torch.float32,)), _stream()))
        return out

    def gather_mean(self, codes, indptr, indices, out=None):
        return self._aggregate(self._lib.bifeat_gather_mean, self._lib.bifeat_gather_mean_i32,
                               codes, indptr, indices, out)

    def gather_sum(self, codes, indptr, indices, out=None):
        return self._aggregate(self._lib.bifeat_gather_sum, self._lib.bifeat_gather_sum_i32,
                               codes, indptr, indices, out)

    def gather_mean_2hop(self, codes, indptr1, indices1, indptr2, indices2, out=None):
        """``bifeat_gather_mean_2hop``: mean over the seed block's lists (entries = destinations
        of the outer block) of the means over the outer block's lists of decoded rows."""
        import torch
        V1, V2 = indptr1.shape[0] - 1, indptr2.shape[0] - 1
        if out is None:
            out = torch.empty((V2, self.D), dtype=torch.float32, device=codes.device)
        elif out.shape != (V2, self.D):
            raise ValueError("out must be [V2, D]")
        i64 = (torch.int64,)
        _check(self._lib.bifeat_gather_mean_2hop(
            self._h, _dev_ptr(codes, (torch.uint8,)), codes.shape[0],
            _dev_ptr(indptr1, i64), _dev_ptr(indices1, i64), V1, indices1.shape[0],
            _dev_ptr(indptr2, i64), _dev_ptr(indices2, i64), V2, indices2.shape[0],
            _dev_ptr(out, (torch.float32,)), _stream()))
        return out

    def poll_status(self, wait: bool = True) -> bool:
        """``bifeat_poll_status``: False if a kernel of an earlier call met a list longer
        than the promised ``mean_max_degree`` (the word is cleared), True otherwise."""
        rc = self._lib.bifeat_poll_status(self._h, _stream(), 1 if wait else 0)
        if rc == EINVAL:
            return False
        _check(rc)
        return True

    def reserve(self, max_requests: int) -> None:
        _check(self._lib.bifeat_reserve(self._h, int(max_requests), _stream()))


def aggregate_rows(x, indptr, indices, out=None, sum: bool = False):
    """``bifeat_aggregate_rows``: mean (or sum) of fp32 rows of ``x`` over CSR lists."""
    import torch
    if x.dim() != 2:
        raise ValueError("x must be [N, D]")
    V, D = indptr.shape[0] - 1, x.shape[1]
    if out is None:
        out = torch.empty((V, D), dtype=torch.float32, device=x.device)
    elif out.shape != (V, D):
        raise ValueError("out must be [V, D]")
    _check(load_library().bifeat_aggregate_rows(
        _dev_ptr(x, (torch.float32,)), x.shape[0], D, _dev_ptr(indptr, (torch.int64,)),
        _dev_ptr(indices, (torch.int64,)), V, indices.shape[0], 1 if sum else 0,
        _dev_ptr(out, (torch.float32,)), _stream()))
    return out


def scale_profile(x, indptr, indices, layers: int, work=None):
    """``bifeat_scale_profile``: mean row length of ``x`` after 0..layers rounds of
    neighbourhood averaging over the whole graph, as a numpy fp64 array."""
    import numpy as np
    import torch
    if x.dim() != 2 or indptr.shape[0] - 1 != x.shape[0]:
        raise ValueError("x must be [N, D] with one list per row")
    N, D = x.shape
    need = min(layers, 2) * N * D
    if work is None and need > 0:
        work = torch.empty(need, dtype=torch.float32, device=x.device)
    elif work is not None and work.numel() < need:
        raise ValueError("work must hold min(layers, 2) * N * D floats")
    scale = np.empty(layers + 1, dtype=np.float64)
    _check(load_library().bifeat_scale_profile(
        _dev_ptr(x, (torch.float32,)), N, D, _dev_ptr(indptr, (torch.int64,)),
        _dev_ptr(indices, (torch.int64,)), indices.shape[0], layers,
        _dev_ptr(work, (torch.float32,)), _np_ptr(scale), _stream()))
    return scale


def check_lists(indptr, indices, N: int) -> bool:
    """``bifeat_check_lists``: True if the CSR lists (``indptr`` may be None for a plain
    index array) satisfy the index contract of the gather calls for a table of N rows."""
    import torch
    V = 0 if indptr is None else indptr.shape[0] - 1
    rc = load_library().bifeat_check_lists(_dev_ptr(indptr, (torch.int64,)), _dev_ptr(indices, (torch.int64,)),
                                           V, indices.shape[0], N, _stream())
    if rc == EINVAL:
        return False
    _check(rc)
    return True
