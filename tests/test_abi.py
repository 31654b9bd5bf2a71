"""The C-ABI library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bifeat.h")


@pytest.fixture(scope="module")
def bf():
    import paper_2207_14696_amd as m
    if not os.path.exists(m.library_path()):
        from paper_2207_14696_amd.build import build
        build()
    m.load_library()
    return m


def test_every_declared_symbol_is_exported(bf):
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    names = set(re.findall(r"\b(bifeat_[a-z_]+)\s*\(", text))
    assert {"bifeat_quantize", "bifeat_gather_dequant", "bifeat_gather_mean", "bifeat_gather_codes",
            "bifeat_fit_update", "bifeat_params_create"} <= names
    lib = C.CDLL(bf.library_path())
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_sizes_and_scheme_validation(bf):
    q = bf.Quantizer(bf.Scheme(bf.UNIFORM, 4), 100)
    assert (q.row_bytes, q.codes_per_row) == (64, 100)
    assert bf.Quantizer(bf.Scheme(bf.UNIFORM, 2), 128).row_bytes == 32
    assert bf.Quantizer(bf.Scheme(bf.LOG, 1), 768).row_bytes == 96
    v = bf.Quantizer(bf.Scheme(bf.VQ, 8, 8, 256), 768)
    assert (v.row_bytes, v.codes_per_row) == (96, 96)
    # more than 256 entries: two bytes per part (Appendix C)
    v2 = bf.Quantizer(bf.Scheme(bf.VQ, 8, 16, 2048, bf.VQ_COSINE), 128)
    assert (v2.row_bytes, v2.codes_per_row) == (16, 8)
    assert bf.Quantizer(bf.Scheme(bf.VQ, 8, 100, 16384), 602).row_bytes == 16
    for bad in [bf.Scheme(bf.UNIFORM, 3), bf.Scheme(bf.LOG, 16), bf.Scheme(bf.VQ, 8, 0, 256),
                bf.Scheme(bf.VQ, 8, 8, 16385), bf.Scheme(bf.VQ, 8, 129, 16),
                bf.Scheme(bf.VQ, 8, 8, 16, 2), bf.Scheme(7, 4)]:
        with pytest.raises(bf.BifeatError) as e:
            bf.Quantizer(bad, 100)
        assert e.value.status == -1
    with pytest.raises(bf.BifeatError):
        bf.Quantizer(bf.Scheme(bf.UNIFORM, 4), 0)


def test_argument_errors_come_before_any_gpu_call(bf):
    lib = bf.load_library()
    q = bf.Quantizer(bf.Scheme(bf.UNIFORM, 4), 16)
    h = q._h
    # null / negative arguments: EINVAL; unfitted parameters: ENOTFIT (no device needed)
    assert lib.bifeat_gather_dequant(h, None, 10, None, 5, None, None) == -1
    assert lib.bifeat_gather_dequant(h, None, 10, None, -1, None, None) == -1
    assert lib.bifeat_gather_mean(h, None, 10, None, None, 3, 7, None, None) == -1
    assert lib.bifeat_quantize(h, None, 0, 4, None, 0, None) == -1
    assert lib.bifeat_quantize(h, None, 9, 0, None, 0, None) == -1           # bad dtype
    assert lib.bifeat_fit_update(h, None, 0, 5, None) == -1
    assert lib.bifeat_gather_dequant(h, 16, 10, 16, 5, 16, None) == -2       # aligned dummies, not fitted
    assert lib.bifeat_gather_dequant(h, 8, 10, 16, 5, 16, None) == -1        # misaligned table
    assert lib.bifeat_aggregate_rows(16, 10, 0, 16, 16, 1, 0, 0, 16, None) == -1     # D = 0
    assert lib.bifeat_aggregate_rows(16, 10, 4, None, 16, 1, 0, 0, 16, None) == -1   # no indptr
    assert lib.bifeat_aggregate_rows(16, 10, 4, 16, 16, 0, 0, 0, 16, None) == 0      # V = 0: no-op
    assert lib.bifeat_scale_profile(16, 10, 4, 16, 16, 5, 65, 16, 16, None) == -1    # too many layers
    assert lib.bifeat_scale_profile(16, 10, 4, 16, 16, 5, 2, None, 16, None) == -1   # no work buffer
    assert lib.bifeat_scale_profile(16, 10, 4, 16, 16, 5, 2, 16, None, None) == -1   # no result array
    assert lib.bifeat_check_lists(None, None, 3, 5, 10, None) == -1                  # no arrays
    assert lib.bifeat_check_lists(16, 16, -1, 5, 10, None) == -1
    # 32-bit list entries, the status query, the workspace calls
    assert lib.bifeat_gather_mean_i32(h, None, 10, None, None, 3, 7, None, None) == -1
    assert lib.bifeat_gather_sum_i32(h, 16, 1 << 31, 16, 16, 1, 1, 16, None) == -1   # ids need 32 bits
    assert lib.bifeat_gather_mean_i32(h, 16, 10, 16, 16, 1, 1, 16, None) == -2       # not fitted
    assert lib.bifeat_gather_mean_2hop(h, None, 10, None, None, 3, 7, None, None, 2, 4, None, None) == -1
    assert lib.bifeat_gather_mean_2hop(h, 16, 10, 16, 16, 3, 7, 16, 16, -2, 4, 16, None) == -1
    assert lib.bifeat_gather_mean_2hop(h, 16, 10, 16, 16, 0, 0, 16, 16, 2, 4, 16, None) == -1  # entries but no outer block
    assert lib.bifeat_gather_mean_2hop(h, 16, 10, 16, 16, 3, 7, 16, 16, 2, 4, 16, None) == -2  # not fitted
    assert lib.bifeat_poll_status(None, None, 0) == -1
    assert lib.bifeat_poll_status(h, None, 0) == 0               # nothing raised, no device touched
    assert lib.bifeat_reserve(None, 5, None) == -1
    assert lib.bifeat_reserve(h, -5, None) == -1
    assert lib.bifeat_reserve(h, 1000, None) == 0                # scalar codes: no workspace
    assert lib.bifeat_gather_dequant_static(h, None, 10, None, 5, None, None) == -1
    assert lib.bifeat_gather_dequant_static(h, 16, 10, 16, 5, 16, None) == -2        # not fitted
    assert lib.bifeat_produce_fit_begin(None, None) == -1
    assert lib.bifeat_produce_fit_end(h, 3) == -1                # no fit open
    assert lib.bifeat_produce_quantize_check(h, 16, 4, 0) == -2  # not fitted
    assert lib.bifeat_set_option(h, b"row_align", 64) == -1      # 16 or 128
    assert lib.bifeat_set_option(h, b"no_such_option", 1) == -1
    assert lib.bifeat_set_option(h, b"mean_slots", 4) == 0
    assert lib.bifeat_row_bytes(None) == -1
    assert lib.bifeat_strerror(-2) == b"quantizer parameters not fitted"
    with pytest.raises(bf.BifeatError):
        q.params_get_uniform()


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2207_14696_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "__init__.py" and "no CPU fallback" in text, f
