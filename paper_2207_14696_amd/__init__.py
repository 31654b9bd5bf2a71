"""MI355X-native feature-loading path of BiFeat (graph feature quantization).

A thin binding over ``libbifeat.so`` (hand-written HIP for gfx950 behind a C
ABI, declared in ``include/bifeat.h``).  PyTorch is used for device memory and
streams only; every step of the path runs in the library's kernels.  There is
no CPU fallback: if the library is missing, loading fails.
"""
from .binding import (Quantizer, Scheme, BifeatError, load_library, library_path,
                      aggregate_rows, scale_profile, check_lists,
                      UNIFORM, LOG, VQ, VQ_L2, VQ_COSINE, F32, F16,
                      OK, EINVAL, ENOTFIT, EHIP, ENOTSUP, ELIMIT, FIT_AGAIN)

__all__ = ["Quantizer", "Scheme", "BifeatError", "load_library", "library_path",
           "aggregate_rows", "scale_profile", "check_lists",
           "UNIFORM", "LOG", "VQ", "VQ_L2", "VQ_COSINE", "F32", "F16",
           "OK", "EINVAL", "ENOTFIT", "EHIP", "ENOTSUP", "ELIMIT", "FIT_AGAIN"]
