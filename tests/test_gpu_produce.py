"""The produced-table interface (include/bifeat_produce.hpp): the library's fit and encode
kernels run over a row source that makes the values inside the kernel - here the synthetic
table's own generator - so that the raw chunk never exists in memory (Sec. 3.3 preprocessing;
Appendix D).  Parameters and packed codes must be those of the chunk entry points and of the
oracle, bit for bit."""
import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk
from helpers import gpu_build_table, scheme_of

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bf():
    import paper_2207_14696_amd as m
    m.load_library()
    return m


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


def _table(spec):
    from bifeat_inputs.device import DeviceTable
    return DeviceTable(spec)


def _produce(q, table, N, pieces, fit=True):
    import torch
    codes = torch.full((N, q.row_bytes), 0xAB, dtype=torch.uint8, device="cuda")
    bounds = np.linspace(0, N, pieces + 1).astype(int)
    if fit:
        q.fit_reset()
        for a, b in zip(bounds[:-1], bounds[1:]):
            table.fit_into(q, int(a), int(b - a))
        assert q.fit_finalize() is False
    for a, b in zip(bounds[:-1], bounds[1:]):
        table.quantize_into(q, codes, int(a), int(b - a))
    torch.cuda.synchronize()
    return codes


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
@pytest.mark.parametrize("D,dtype", [(100, "f32"), (128, "f16"), (37, "f32"), (37, "f16"), (768, "f16")])
def test_uniform_codes_from_a_produced_table(bf, torch, bits, D, dtype):
    spec = FeatureSpec(5003, D, 3, dtype)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, bits)
    want = orc.pack(orc.uniform_encode(x, bits, mn, inv), bits)
    q = bf.Quantizer(scheme_of("uniform", bits), D)
    got = _produce(q, _table(spec), spec.N, 3)
    gmn, gmx, gscale, ginv = q.params_get_uniform()
    for a, b in [(gmn, mn), (gmx, mx), (gscale, scale), (ginv, inv)]:
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(got.cpu().numpy(), want)
    # the chunk entry points give the same table
    q2 = bf.Quantizer(scheme_of("uniform", bits), D)
    assert torch.equal(gpu_build_table(q2, _table(spec), spec.N, 2000), got)
    # line-aligned layout too
    q3 = bf.Quantizer(scheme_of("uniform", bits), D, row_align=128)
    q3.params_set_uniform(mn, mx)
    got3 = _produce(q3, _table(spec), spec.N, 2, fit=False).cpu().numpy()
    assert np.array_equal(got3[:, :want.shape[1]], want) and not got3[:, want.shape[1]:].any()


@pytest.mark.parametrize("bits,D,dtype", [(1, 768, "f16"), (2, 100, "f32"), (4, 37, "f32"), (8, 64, "f16")])
def test_log_codes_from_a_produced_table(bf, torch, bits, D, dtype):
    spec = FeatureSpec(4001, D, 5, dtype)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    e_min, e_max = orc.log_range(orc.log_fit(x))
    T, V = orc.log_tables(e_min, e_max, bits)
    want = orc.pack(orc.log_encode(x, bits, T), bits)
    q = bf.Quantizer(scheme_of("log", bits), D)
    got = _produce(q, _table(spec), spec.N, 4)
    assert q.params_get_log()[:2] == (e_min, e_max)
    assert np.array_equal(got.cpu().numpy(), want)


def test_chunks_and_produced_pieces_mix_in_one_fit(bf, torch):
    spec = FeatureSpec(3000, 64, 7)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    t = _table(spec)
    q = bf.Quantizer(scheme_of("uniform", 4), 64)
    q.fit_reset()
    t.fit_into(q, 0, 1000)
    q.fit_update(t.chunk(1000, 1000))
    t.fit_into(q, 2000, 1000)
    q.fit_finalize()
    mn, mx = orc.fit_minmax(x)
    gmn, gmx, _, _ = q.params_get_uniform()
    assert np.array_equal(gmn, mn) and np.array_equal(gmx, mx)


def test_produced_interface_refuses_what_it_does_not_cover(bf, torch):
    lib = bf.load_library()
    v = bf.Quantizer(scheme_of("vq", 8, 8, 16), 64)
    assert lib.bifeat_produce_fit_begin(v._h, None) == bf.ENOTSUP
    assert lib.bifeat_produce_quantize_check(v._h, 16, 4, 0) == bf.ENOTSUP
    lq = bf.Quantizer(scheme_of("log", 2), 64)
    lq.fit_set_log_clip(0.01)
    assert lib.bifeat_produce_fit_begin(lq._h, None) == bf.ENOTSUP
    u = bf.Quantizer(scheme_of("uniform", 4), 64)
    assert lib.bifeat_produce_quantize_check(u._h, 16, 4, 0) == bf.ENOTFIT
    assert lib.bifeat_produce_fit_end(u._h, 5) == bf.EINVAL          # no fit open
    assert lib.bifeat_produce_fit_begin(u._h, None) == bf.OK
    assert lib.bifeat_produce_fit_end(u._h, -1) == bf.EINVAL
    assert lib.bifeat_produce_quantize_check(u._h, 8, 4, 0) == bf.EINVAL   # misaligned table
