"""Device side of the feature generator: fills chunks of the synthetic table in
GPU memory with ``csrc/synth.hip`` (same recipe as ``features.py``, bit for
bit), so that tables of hundreds of GB can be streamed through the quantizer
without ever existing on the host."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

from .features import C_Z, FeatureSpec, column_params, stream_key, STREAM_FEAT

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "synth.hip")
_SO = os.path.join(_HERE, "libbifeat_synth.so")
_SRC_FUSED = os.path.join(_HERE, "csrc", "synth_fused.hip")
_SO_FUSED = os.path.join(_HERE, "libbifeat_synth_fused.so")
_ROOT = os.path.dirname(_HERE)
_lib = None
_lib_fused = None


def build() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = _SO + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                           "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                           "-o", tmp, _SRC])
    os.replace(tmp, _SO)
    # the generator as a row source of the library's produced-table interface: the library's
    # kernel templates instantiated for it (needs libbifeat.so built first, for linking)
    pkg = os.path.join(_ROOT, "paper_2207_14696_amd")
    tmp = _SO_FUSED + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                           "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                           "-I", os.path.join(_ROOT, "include"), "-I", os.path.join(pkg, "csrc"),
                           "-o", tmp, _SRC_FUSED, "-L", pkg, "-lbifeat",
                           "-Wl,-rpath,$ORIGIN/../paper_2207_14696_amd"])
    os.replace(tmp, _SO_FUSED)
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise ImportError(f"{_SO} is missing: build it with bifeat_inputs.device.build()")
        _lib = C.CDLL(_SO)
        _lib.bifeat_synth_fill.restype = C.c_int
        _lib.bifeat_synth_fill.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int,
                                           C.c_uint64, C.c_float, C.c_void_p, C.c_void_p,
                                           C.c_void_p]
    return _lib


def _load_fused():
    global _lib_fused
    if _lib_fused is None:
        if not os.path.exists(_SO_FUSED):
            raise ImportError(f"{_SO_FUSED} is missing: build it with bifeat_inputs.device.build()")
        _lib_fused = C.CDLL(_SO_FUSED)
        common = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_uint64, C.c_float,
                  C.c_void_p, C.c_void_p]
        _lib_fused.bifeat_synth_fit.restype = C.c_int
        _lib_fused.bifeat_synth_fit.argtypes = common + [C.c_void_p]
        _lib_fused.bifeat_synth_quantize.restype = C.c_int
        _lib_fused.bifeat_synth_quantize.argtypes = common + [C.c_void_p, C.c_void_p]
    return _lib_fused


class DeviceTable:
    """Streams chunks of the table described by ``spec`` into CUDA tensors."""

    def __init__(self, spec: FeatureSpec, device="cuda"):
        import torch
        self.spec = spec
        self.device = device
        mu, sigma = column_params(spec.seed, spec.D)
        self.mu = torch.from_numpy(mu).to(device)
        self.sigma = torch.from_numpy(sigma).to(device)
        self.key = int(stream_key(spec.seed, STREAM_FEAT))
        self.torch_dtype = torch.float32 if spec.dtype == "f32" else torch.float16

    def chunk(self, row0: int, rows: int, out=None):
        import torch
        if out is None:
            out = torch.empty((rows, self.spec.D), dtype=self.torch_dtype, device=self.device)
        assert out.is_contiguous() and out.shape == (rows, self.spec.D) and out.dtype == self.torch_dtype
        rc = _load().bifeat_synth_fill(out.data_ptr(), 0 if self.spec.dtype == "f32" else 1,
                                       row0, rows, self.spec.D, self.key, float(C_Z),
                                       self.mu.data_ptr(), self.sigma.data_ptr(),
                                       torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError(f"bifeat_synth_fill: hip error {rc}")
        return out

    # ---- the table as a row source of the library's kernels: nothing but codes is written
    def _fused_args(self, q, row0: int, rows: int):
        return [q._h, 0 if self.spec.dtype == "f32" else 1, row0, rows, self.spec.D, self.key,
                float(C_Z), self.mu.data_ptr(), self.sigma.data_ptr()]

    def fit_into(self, q, row0: int, rows: int) -> None:
        """Streaming fit of quantizer ``q`` over rows [row0, row0+rows), produced in the kernel."""
        import torch
        rc = _load_fused().bifeat_synth_fit(*self._fused_args(q, row0, rows),
                                            torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError(f"bifeat_synth_fit: status {rc}")

    def quantize_into(self, q, codes, row0: int, rows: int) -> None:
        """Encode + pack rows [row0, row0+rows) into the same rows of the packed table ``codes``."""
        import torch
        assert codes.dtype == torch.uint8 and codes.is_contiguous() and codes.shape[1] == q.row_bytes
        assert 0 <= row0 and row0 + rows <= codes.shape[0]
        rc = _load_fused().bifeat_synth_quantize(*self._fused_args(q, row0, rows), codes.data_ptr(),
                                                 torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError(f"bifeat_synth_quantize: status {rc}")
