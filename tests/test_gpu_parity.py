"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on
the same seeded inputs.  Codes, packed rows and fitted parameters are compared
bit for bit; decoded values and means to 1e-5 relative (see helpers.assert_close).
Sizes span several workgroup tiles and a ragged tail."""
import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk
from helpers import (assert_close, gpu_build_table, oracle_uniform_table, random_csr, scheme_of)

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


def _dev_table(spec):
    from bifeat_inputs.device import DeviceTable
    return DeviceTable(spec)


@pytest.mark.parametrize("D,dtype", [(100, "f32"), (128, "f16"), (37, "f32"), (37, "f16"), (768, "f16")])
def test_device_generator_is_bit_identical(torch, D, dtype):
    spec = FeatureSpec(5003, D, 0, dtype)
    got = _dev_table(spec).chunk(1000, 4003).cpu().numpy()
    want = feature_chunk(spec, 1000, 4003)
    assert got.dtype == want.dtype and np.array_equal(got.view(np.uint8), want.view(np.uint8))


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
@pytest.mark.parametrize("D,dtype", [(100, "f32"), (128, "f32"), (37, "f32"), (200, "f16")])
def test_uniform_fit_and_codes_bit_exact(bf, torch, bits, D, dtype):
    spec = FeatureSpec(9001, D, 1, dtype)
    x, (mn, mx, scale, inv), s, codes = oracle_uniform_table(spec, bits)
    q = bf.Quantizer(scheme_of("uniform", bits), D)
    assert q.row_bytes == s.row_bytes
    got = gpu_build_table(q, _dev_table(spec), spec.N, 2500)     # 4 chunks, ragged last
    gmn, gmx, gscale, ginv = q.params_get_uniform()
    for a, b in [(gmn, mn), (gmx, mx), (gscale, scale), (ginv, inv)]:
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(got.cpu().numpy(), codes)


def test_uniform_params_set_matches_fit(bf, torch):
    spec = FeatureSpec(3000, 64, 2)
    x, (mn, mx, scale, inv), s, codes = oracle_uniform_table(spec, 4)
    q = bf.Quantizer(scheme_of("uniform", 4), 64)
    q.params_set_uniform(mn, mx)
    _, _, gscale, ginv = q.params_get_uniform()
    assert np.array_equal(gscale, scale) and np.array_equal(ginv, inv)
    got = gpu_build_table(q, _dev_table(spec), spec.N, 3000, fit=False)
    assert np.array_equal(got.cpu().numpy(), codes)


def test_uniform_special_values(bf, torch):
    # constant column, NaN, out-of-range values, exact ties
    D = 8
    x = feature_chunk(FeatureSpec(600, D, 3), 0, 600).copy()
    x[:, 2] = 0.25
    x[5, 0] = np.nan
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, 4)
    q = bf.Quantizer(scheme_of("uniform", 4), D)
    xt = torch.from_numpy(x).cuda()
    q.fit_update(xt)
    q.fit_finalize()
    gmn, gmx, gscale, ginv = q.params_get_uniform()
    assert np.array_equal(gmn, mn) and np.array_equal(gmx, mx) and gscale[2] == 0 and ginv[2] == 0
    y = x.copy()
    y[0, :] = 1e9
    y[1, :] = -1e9
    y[2, :] = (mn + 2.5 * scale).astype(np.float32)           # near ties
    codes = torch.zeros((600, q.row_bytes), dtype=torch.uint8, device="cuda")
    q.quantize(torch.from_numpy(y).cuda(), codes, 0)
    want = orc.pack(orc.uniform_encode(y, 4, mn, inv), 4)
    assert np.array_equal(codes.cpu().numpy(), want)


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_log_fit_and_codes_bit_exact(bf, torch, k):
    D = 52
    spec = FeatureSpec(7001, D, 4)
    x = feature_chunk(spec, 0, spec.N)
    st = orc.log_fit(x)
    e_min, e_max = orc.log_range(st)
    T, V = orc.log_tables(e_min, e_max, k)
    want = orc.pack(orc.log_encode(x, k, T), k)
    q = bf.Quantizer(scheme_of("log", k), D)
    got = gpu_build_table(q, _dev_table(spec), spec.N, 3000)
    ge_min, ge_max, gT, gV = q.params_get_log()
    assert (ge_min, ge_max) == (e_min, e_max)
    assert np.array_equal(gT, T) and np.array_equal(gV, V)
    assert np.array_equal(got.cpu().numpy(), want)
    # a clipped range supplied by the caller (oracle: exact order statistics)
    c_min, c_max = orc.log_range_clipped(x, 0.02)
    T, V = orc.log_tables(c_min, c_max, k)
    q.params_set_log(c_min, c_max)
    got = gpu_build_table(q, _dev_table(spec), spec.N, 7001, fit=False)
    assert np.array_equal(got.cpu().numpy(), orc.pack(orc.log_encode(x, k, T), k))


def test_log_zero_and_sign_handling(bf, torch):
    x = np.array([[0.0, -0.0, 1.0, -1.0, np.nan, 3.0, -2.0, 0.5]], np.float32)
    q = bf.Quantizer(scheme_of("log", 2), 8)
    q.params_set_log(-1.0, 2.0)
    T, _ = orc.log_tables(-1.0, 2.0, 2)
    codes = torch.zeros((1, q.row_bytes), dtype=torch.uint8, device="cuda")
    q.quantize(torch.from_numpy(x).cuda(), codes, 0)
    assert np.array_equal(codes.cpu().numpy(), orc.pack(orc.log_encode(x, 2, T), 2))


@pytest.mark.parametrize("D,w,length,dtype", [(64, 8, 256, "f32"), (96, 4, 16, "f16"),
                                              (23, 5, 7, "f32"), (40, 16, 64, "f32"),
                                              (12, 1, 4, "f32")])
def test_vq_codes_bit_exact(bf, torch, D, w, length, dtype):
    spec = FeatureSpec(4099, D, 5, dtype)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    cb, _ = orc.vq_train(x[:1500], w, length, iters=4)
    want = orc.pack(orc.vq_assign(x, w, cb), 8)
    q = bf.Quantizer(scheme_of("vq", 8, w, length), D)
    q.params_set_codebooks(cb)
    assert np.array_equal(q.params_get_codebooks(), cb)
    got = gpu_build_table(q, _dev_table(spec), spec.N, 1700, fit=False)
    assert np.array_equal(got.cpu().numpy(), want)


def _tables(bf, torch, kind, bits, D, N=6007, w=8, length=32, seed=6):
    """(quantizer, oracle scheme, packed codes as numpy + as CUDA tensor)."""
    spec = FeatureSpec(N, D, seed)
    x = feature_chunk(spec, 0, N)
    if kind == "uniform":
        _, (mn, mx, scale, inv), s, codes = oracle_uniform_table(spec, bits)
        q = bf.Quantizer(scheme_of("uniform", bits), D)
        q.params_set_uniform(mn, mx)
    elif kind == "log":
        e_min, e_max = orc.log_range_clipped(x, 0.01)
        T, V = orc.log_tables(e_min, e_max, bits)
        s = orc.Scheme.log(D, V, bits)
        codes = orc.pack(orc.log_encode(x, bits, T), bits)
        q = bf.Quantizer(scheme_of("log", bits), D)
        q.params_set_log(e_min, e_max)
    else:
        cb, _ = orc.vq_train(x[:1000], w, length, iters=3)
        s = orc.Scheme.vq(D, cb)
        codes = orc.pack(orc.vq_assign(x, w, cb), 8)
        q = bf.Quantizer(scheme_of("vq", 8, w, length), D)
        q.params_set_codebooks(cb)
    return q, s, codes, torch.from_numpy(codes).cuda()


CASES = [("uniform", 1, 768), ("uniform", 2, 128), ("uniform", 4, 100), ("uniform", 8, 128),
         ("uniform", 4, 37), ("uniform", 8, 5), ("uniform", 1, 70), ("uniform", 2, 1),
         ("log", 1, 64), ("log", 1, 768), ("log", 2, 100), ("log", 4, 37), ("log", 8, 16),
         ("log", 4, 128), ("log", 4, 100), ("log", 4, 768), ("log", 8, 200), ("log", 8, 1024),
         ("vq", 8, 64), ("vq", 8, 100), ("vq", 8, 23), ("vq", 8, 96)]


@pytest.mark.parametrize("kind,bits,D", CASES)
def test_gather_codes_and_dequant(bf, torch, kind, bits, D):
    w = {23: 5, 100: 4, 96: 16}.get(D, 8)
    q, s, codes, dcodes = _tables(bf, torch, kind, bits, D, w=w)
    rng = np.random.default_rng(0)
    idx = rng.integers(0, codes.shape[0], 3001).astype(np.int64)
    idx[:3] = [0, codes.shape[0] - 1, 0]
    didx = torch.from_numpy(idx).cuda()
    assert np.array_equal(q.gather_codes(dcodes, didx).cpu().numpy(), orc.gather_codes(codes, idx))
    want = orc.gather_dequant(s, codes, idx)
    assert_close(q.gather_dequant(dcodes, didx).cpu().numpy(), want, s, "gather_dequant")
    if kind != "vq":            # both forms of the scalar kernel (LDS-staged tiles / flat)
        q.set_option("dequant_flat", 1)
        assert_close(q.gather_dequant(dcodes, didx).cpu().numpy(), want, s, "gather_dequant flat")
        q.set_option("dequant_flat", 0)
    else:                       # codebooks from L2 instead of LDS-resident slices
        q.set_option("vq_sliced", 0)
        assert_close(q.gather_dequant(dcodes, didx).cpu().numpy(), want, s, "gather_dequant L2 tiles")
        q.set_option("dequant_flat", 1)
        assert_close(q.gather_dequant(dcodes, didx).cpu().numpy(), want, s, "gather_dequant L2 flat")
        q.set_option("dequant_flat", 0)
        q.set_option("vq_sliced", 1)
    # empty request
    empty = torch.empty(0, dtype=torch.int64, device="cuda")
    assert q.gather_dequant(dcodes, empty).shape == (0, D)
    assert q.gather_codes(dcodes, empty).shape == (0, q.row_bytes)


@pytest.mark.parametrize("kind,bits,D", CASES)
def test_gather_mean(bf, torch, kind, bits, D):
    w = {23: 5, 100: 4, 96: 16}.get(D, 8)
    q, s, codes, dcodes = _tables(bf, torch, kind, bits, D, w=w)
    rng = np.random.default_rng(1)
    # long lists cross the integer-accumulator capacity of every bit width
    # (64 / 65: either side of the look-up kernel's limit for 4- and 8-bit logarithmic codes)
    hubs = (90, 300, 700, 4500) if kind == "uniform" else (40, 64, 65, 300)
    indptr, indices = random_csr(1501, codes.shape[0], 30, rng, hubs=hubs)
    want = orc.gather_mean(s, codes, indptr, indices)
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    got = q.gather_mean(dcodes, dptr, dind).cpu().numpy()
    assert not got[0].any()
    assert_close(got, want, s, "gather_mean")
    if kind == "log":
        q.set_option("mean_generic", 1)
        assert_close(q.gather_mean(dcodes, dptr, dind).cpu().numpy(), want, s, "general kernel only")
        q.set_option("mean_generic", 0)
    if kind == "uniform":
        for slots in (1, 2, 8, 64):
            q.set_option("mean_slots", slots)
            assert_close(q.gather_mean(dcodes, dptr, dind).cpu().numpy(), want, s, f"slots={slots}")
        q.set_option("mean_slots", 0)
        q.set_option("mean_generic", 1)
        assert_close(q.gather_mean(dcodes, dptr, dind).cpu().numpy(), want, s, "generic")
        q.set_option("mean_generic", 0)
    if kind == "vq":
        q.set_option("vq_sliced", 0)
        assert_close(q.gather_mean(dcodes, dptr, dind).cpu().numpy(), want, s, "L2 codebooks")
        q.set_option("vq_sliced", 1)


def test_gather_mean_degenerate_blocks(bf, torch):
    q, s, codes, dcodes = _tables(bf, torch, "uniform", 4, 100)
    z = torch.zeros(1, dtype=torch.int64, device="cuda")
    assert q.gather_mean(dcodes, z, torch.empty(0, dtype=torch.int64, device="cuda")).shape == (0, 100)
    # every list empty
    ptr = torch.zeros(18, dtype=torch.int64, device="cuda")
    out = q.gather_mean(dcodes, ptr, torch.empty(0, dtype=torch.int64, device="cuda"))
    assert out.shape == (17, 100) and not out.any()
    # one destination, one neighbour: equals that row's dequantization
    ptr = torch.tensor([0, 1], dtype=torch.int64, device="cuda")
    ind = torch.tensor([77], dtype=torch.int64, device="cuda")
    one = q.gather_mean(dcodes, ptr, ind).cpu().numpy()
    assert_close(one, orc.gather_dequant(s, codes, np.array([77])), s)


def test_wide_rows_take_several_passes(bf, torch):
    # 8-bit codes, D = 1500: a packed row is longer than one wavefront's 64 x 16 bytes
    q, s, codes, dcodes = _tables(bf, torch, "uniform", 8, 1500, N=301)
    rng = np.random.default_rng(2)
    indptr, indices = random_csr(97, 301, 12, rng, hubs=(300,))
    got = q.gather_mean(dcodes, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda())
    assert_close(got.cpu().numpy(), orc.gather_mean(s, codes, indptr, indices), s)
    idx = rng.integers(0, 301, 200).astype(np.int64)
    got = q.gather_dequant(dcodes, torch.from_numpy(idx).cuda()).cpu().numpy()
    assert_close(got, orc.gather_dequant(s, codes, idx), s)


def test_argument_errors(bf, torch):
    q = bf.Quantizer(scheme_of("uniform", 4), 16)
    codes = torch.zeros((4, q.row_bytes), dtype=torch.uint8, device="cuda")
    idx = torch.zeros(2, dtype=torch.int64, device="cuda")
    with pytest.raises(bf.BifeatError) as e:
        q.gather_dequant(codes, idx)
    assert e.value.status == -2                       # not fitted
    with pytest.raises(bf.BifeatError) as e:
        q.fit_finalize()
    assert e.value.status == -2
    v = bf.Quantizer(scheme_of("vq", 8, 4, 16), 16)
    with pytest.raises(bf.BifeatError) as e:
        v.fit_update(torch.zeros((3, 16), device="cuda"))
    assert e.value.status == -1                       # fewer sample rows than codebook entries


@pytest.mark.parametrize("kind,bits,D", [("uniform", 1, 768), ("uniform", 2, 128), ("uniform", 4, 100),
                                         ("uniform", 8, 128), ("uniform", 4, 768), ("uniform", 1, 64),
                                         ("uniform", 8, 4), ("log", 2, 128), ("log", 1, 256), ("log", 4, 128)])
def test_gather_mean_short_lists_take_two_kernels(bf, torch, kind, bits, D):
    # sampled-block shape: short lists (the short-list kernel, chosen on the average length)
    # with longer ones mixed in: up to 64 they go to the short-list kernel's wide form where
    # there is one (15 / 17 are the narrow forms' capacities), beyond that to the general
    # kernel; each launch skips the others' destinations
    q, s, codes, dcodes = _tables(bf, torch, kind, bits, D, N=4001)
    rng = np.random.default_rng(3)
    indptr, indices = random_csr(2307, codes.shape[0], 10, rng, hubs=(15, 16, 17, 18, 40, 64, 65, 300))
    want = orc.gather_mean(s, codes, indptr, indices)
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    out = torch.full((2307, D), float("nan"), device="cuda")
    q.gather_mean(dcodes, dptr, dind, out)
    assert_close(out.cpu().numpy(), want, s, "lean + general")
    q.set_option("mean_lean", 0)
    assert_close(q.gather_mean(dcodes, dptr, dind).cpu().numpy(), want, s, "general only")
    q.set_option("mean_lean", 1)
    # all lists short and the caller says so: the lean kernel alone
    indptr, indices = random_csr(1000, codes.shape[0], 5, rng)
    want = orc.gather_mean(s, codes, indptr, indices)
    q.set_option("mean_max_degree", 5)
    out = torch.full((1000, D), float("nan"), device="cuda")
    q.gather_mean(dcodes, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), out)
    assert_close(out.cpu().numpy(), want, s, "lean only")
    q.set_option("mean_max_degree", 0)


@pytest.mark.parametrize("D,w,length,dtype", [(64, 8, 256, "f32"), (96, 4, 16, "f16"), (23, 5, 7, "f32")])
def test_vq_codebook_training_matches_oracle_distortion(bf, torch, D, w, length, dtype):
    # Lloyd k-means on the GPU from the same start as the oracle's: judged on
    # distortion (fp32 atomic sums are not bit-reproducible), and every round must
    # not increase it
    spec = FeatureSpec(6000, D, 9, dtype)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    sample, held = x[:4000], x[4000:]
    ocb, odist = orc.vq_train(sample, w, length, iters=10)
    q = bf.Quantizer(scheme_of("vq", 8, w, length), D)
    q.fit_update(_dev_table(spec).chunk(0, 4000))
    q.fit_finalize()
    gcb = q.params_get_codebooks()
    gdist = q.vq_distortion(10)
    assert np.isfinite(gcb).all()
    assert np.all(np.diff(gdist) <= 1e-4 * gdist[0])
    assert np.allclose(gdist, odist, rtol=2e-3)        # same trajectory as the oracle

    def distortion(cb):
        s = orc.Scheme.vq(D, cb)
        dec = orc.gather_dequant(s, orc.pack(orc.vq_assign(held, w, cb), 8), np.arange(len(held)))
        return ((dec.astype(np.float64) - held) ** 2).sum(1).mean()
    assert distortion(gcb) <= 1.01 * distortion(ocb)
    # a table encoded with the trained codebooks: codes equal the oracle's for those codebooks
    codes = gpu_build_table(q, _dev_table(spec), spec.N, 2500, fit=False)
    assert np.array_equal(codes.cpu().numpy(), orc.pack(orc.vq_assign(x, w, gcb), 8))


# ------------------------------------- vector-code variants: cosine metric, two-byte indices
VQ_VARIANTS = [(64, 16, 2048, "l2", "f32"), (48, 16, 600, "cosine", "f32"),
               (207, 100, 300, "l2", "f32"), (64, 8, 64, "cosine", "f16"),
               (40, 5, 7, "cosine", "f32"), (70, 40, 20, "cosine", "f32")]


@pytest.mark.parametrize("D,w,length,metric,dtype", VQ_VARIANTS)
def test_vq_variant_codes_bit_exact(bf, torch, D, w, length, metric, dtype):
    spec = FeatureSpec(3001, D, 15, dtype)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    cb, _ = orc.vq_train(x[:max(length, 800)], w, length, iters=2, metric=metric)
    bits = orc.vq_code_bits(length)
    want = orc.pack(orc.vq_assign(x, w, cb, metric=metric), bits)
    q = bf.Quantizer(scheme_of("vq", 8, w, length, metric), D)
    assert q.row_bytes == want.shape[1]
    q.params_set_codebooks(cb)
    got = gpu_build_table(q, _dev_table(spec), spec.N, 1300, fit=False)
    assert np.array_equal(got.cpu().numpy(), want)


@pytest.mark.parametrize("D,w,length", [(64, 8, 700), (100, 4, 1000), (46, 23, 300)])
def test_two_byte_codes_gather(bf, torch, D, w, length):
    spec = FeatureSpec(5003, D, 16)
    x = feature_chunk(spec, 0, spec.N)
    cb, _ = orc.vq_train(x[:1200], w, length, iters=2)
    s = orc.Scheme.vq(D, cb)
    codes = orc.pack(orc.vq_assign(x, w, cb), 16)
    q = bf.Quantizer(scheme_of("vq", 8, w, length), D)
    q.params_set_codebooks(cb)
    dcodes = torch.from_numpy(codes).cuda()
    rng = np.random.default_rng(3)
    idx = rng.integers(0, spec.N, 2001).astype(np.int64)
    didx = torch.from_numpy(idx).cuda()
    assert np.array_equal(q.gather_codes(dcodes, didx).cpu().numpy(), orc.gather_codes(codes, idx))
    assert_close(q.gather_dequant(dcodes, didx).cpu().numpy(), orc.gather_dequant(s, codes, idx), s)
    indptr, indices = random_csr(901, spec.N, 20, rng, hubs=(200,))
    got = q.gather_mean(dcodes, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda())
    assert_close(got.cpu().numpy(), orc.gather_mean(s, codes, indptr, indices), s, "gather_mean")


@pytest.mark.parametrize("D,w,length,metric", [(64, 8, 32, "cosine"), (32, 4, 512, "l2"),
                                               (60, 20, 300, "cosine")])
def test_vq_variant_training_matches_oracle_distortion(bf, torch, D, w, length, metric):
    spec = FeatureSpec(6000, D, 17)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    sample, held = x[:4000], x[4000:]
    ocb, odist = orc.vq_train(sample, w, length, iters=6, metric=metric)
    if metric == "l2":      # the metric entry reports distortion the same way for both metrics
        odist = orc.vq_train(sample, w, length, iters=6)[1]
    q = bf.Quantizer(scheme_of("vq", 8, w, length, metric), D)
    q.set_option("vq_iters", 6)
    q.fit_update(_dev_table(spec).chunk(0, 4000))
    q.fit_finalize()
    gcb = q.params_get_codebooks()
    gdist = q.vq_distortion(6)
    assert np.isfinite(gcb).all()
    # same trajectory as the oracle's (fp32 atomic sums against fp64 means: measured agreement
    # is ~5e-7 relative; the bounds are those of the one-byte Euclidean trainer's test)
    assert np.allclose(gdist, odist, rtol=2e-3)
    bits = orc.vq_code_bits(length)

    def distortion(cb):
        s = orc.Scheme.vq(D, cb)
        dec = orc.gather_dequant(s, orc.pack(orc.vq_assign(held, w, cb, metric=metric), bits),
                                 np.arange(len(held)))
        return ((dec.astype(np.float64) - held) ** 2).sum(1).mean()
    assert distortion(gcb) <= 1.01 * distortion(ocb)
    codes = gpu_build_table(q, _dev_table(spec), spec.N, 2500, fit=False)
    assert np.array_equal(codes.cpu().numpy(),
                          orc.pack(orc.vq_assign(x, w, gcb, metric=metric), bits))


# ---------------------------------------------- clipped logarithmic range fitted on the GPU
@pytest.mark.parametrize("D,dtype,frac,chunk", [(37, "f32", 0.01, 700), (128, "f16", 0.001, 1024),
                                                (64, "f32", 0.25, 5000), (5, "f32", 0.0625, 333)])
def test_clipped_log_range_is_the_exact_order_statistic(bf, torch, D, dtype, frac, chunk):
    spec = FeatureSpec(5000, D, 21, dtype)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    want = orc.log_range_clipped(x, frac)
    q = bf.Quantizer(scheme_of("log", 2), D)
    q.fit_set_log_clip(frac)
    table = _dev_table(spec)
    passes = 0
    again = True
    q.fit_reset()
    while again:
        for r0 in range(0, spec.N, chunk):
            q.fit_update(table.chunk(r0, min(chunk, spec.N - r0)))
        again = q.fit_finalize()
        passes += 1
    assert passes == 3
    e_min, e_max, T, V = q.params_get_log()
    assert (e_min, e_max) == want                 # same magnitudes, same log2
    oT, oV = orc.log_tables(*want, 2)
    assert np.array_equal(T, oT) and np.array_equal(V, oV)
    codes = gpu_build_table(q, table, spec.N, 1700, fit=False)
    assert np.array_equal(codes.cpu().numpy(), orc.pack(orc.log_encode(x, 2, oT), 2))


def test_clipped_log_fit_special_values_and_errors(bf, torch):
    x = np.zeros((64, 8), np.float32)
    x[3, 2], x[5, 5], x[7, 1], x[9, 9 % 8] = np.inf, np.nan, -3.5, 0.25
    x[20:40] = np.linspace(-2, 2, 160, dtype=np.float32).reshape(20, 8)
    want = orc.log_range_clipped(x, 0.1)
    q = bf.Quantizer(scheme_of("log", 4), 8)
    q.fit_set_log_clip(0.1)
    dx = torch.from_numpy(x).cuda()
    q.fit_reset()
    for _ in range(3):
        q.fit_update(dx)
        again = q.fit_finalize()
    assert not again
    e_min, e_max, _, _ = q.params_get_log()
    assert (e_min, e_max) == want
    # a table of zeros: no magnitudes to rank, range (0, 0) after the first pass
    q.fit_reset()
    q.fit_update(torch.zeros((10, 8), device="cuda"))
    assert q.fit_finalize() is False
    assert q.params_get_log()[:2] == (0.0, 0.0)
    # different data in a later pass is refused
    q.fit_reset()
    q.fit_update(dx)
    assert q.fit_finalize() is True
    q.fit_update(torch.zeros((64, 8), device="cuda"))
    with pytest.raises(bf.BifeatError):
        q.fit_finalize()
    with pytest.raises(bf.BifeatError):
        q.fit_set_log_clip(0.5)


# ------------------------------------------------------------------- sum aggregator
def _assert_sum_close(got, want, s, n, what=""):
    """|gpu - oracle| <= 1e-5 * max(|oracle|, n_v * A_j): a sum of n_v terms of size A_j."""
    from helpers import column_magnitude, REL_TOL
    A = column_magnitude(s).astype(np.float64)[None, :] * np.maximum(n, 1)[:, None]
    bound = REL_TOL * np.maximum(np.abs(want.astype(np.float64)), A)
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    assert not (err > bound).any(), f"{what}: worst err/bound = {(err / bound).max():.3g}"


@pytest.mark.parametrize("kind,bits,D", CASES)
def test_gather_sum(bf, torch, kind, bits, D):
    w = {23: 5, 100: 4, 96: 16}.get(D, 8)
    q, s, codes, dcodes = _tables(bf, torch, kind, bits, D, w=w)
    rng = np.random.default_rng(2)
    hubs = (90, 300, 700, 4500) if kind == "uniform" else (300,)
    indptr, indices = random_csr(1201, codes.shape[0], 30, rng, hubs=hubs)
    want = orc.gather_sum(s, codes, indptr, indices)
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    got = q.gather_sum(dcodes, dptr, dind).cpu().numpy()
    assert not got[0].any()
    _assert_sum_close(got, want, s, np.diff(indptr), "gather_sum")
    # the mean entry point is unaffected by a sum call before it
    assert_close(q.gather_mean(dcodes, dptr, dind).cpu().numpy(), orc.gather_mean(s, codes, indptr, indices), s)
    # short lists with the caller's bound: the short-list kernels alone
    indptr, indices = random_csr(801, codes.shape[0], 10, rng)
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    q.set_option("mean_max_degree", 10)
    got = q.gather_sum(dcodes, dptr, dind).cpu().numpy()
    q.set_option("mean_max_degree", 0)
    _assert_sum_close(got, orc.gather_sum(s, codes, indptr, indices), s, np.diff(indptr), "short lists")


def test_mean_with_self_loops_on_the_gpu(bf, torch):
    # D^-1 (A + I) of Appendix A.1: the destination listed among its own neighbours
    q, s, codes, dcodes = _tables(bf, torch, "uniform", 4, 100)
    rng = np.random.default_rng(8)
    V, N = 700, codes.shape[0]
    dst_rows = rng.choice(N, V, replace=False)
    deg = rng.integers(0, 12, V)
    ptr = np.concatenate([[0], np.cumsum(deg + 1)]).astype(np.int64)
    idx = rng.integers(0, N, ptr[-1]).astype(np.int64)
    idx[ptr[1:] - 1] = dst_rows                      # last entry of every list: the destination
    got = q.gather_mean(dcodes, torch.from_numpy(ptr).cuda(), torch.from_numpy(idx).cuda())
    assert_close(got.cpu().numpy(), orc.gather_mean(s, codes, ptr, idx), s)


@pytest.mark.parametrize("kind,bits,D", [("uniform", 4, 100), ("vq", 8, 64), ("log", 2, 100), ("log", 4, 128)])
def test_calls_replay_from_a_captured_graph(bf, torch, kind, bits, D):
    # the per-iteration calls enqueue kernels only (no memset, no synchronisation, no
    # allocation once the vector-code scratch has its size), so a step can be captured once
    # and replayed; every replay must reproduce the eager result, with eager work in between
    q, s, codes, dcodes = _tables(bf, torch, kind, bits, D)
    rng = np.random.default_rng(12)
    idx = torch.from_numpy(rng.integers(0, codes.shape[0], 1500).astype(np.int64)).cuda()
    indptr, indices = random_csr(400, codes.shape[0], 10, rng, hubs=(120,))
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    eager_a = q.gather_dequant(dcodes, idx).clone()
    eager_b = q.gather_mean(dcodes, dptr, dind).clone()
    out_a, out_b = torch.empty_like(eager_a), torch.empty_like(eager_b)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        q.gather_dequant(dcodes, idx, out_a)
        q.gather_mean(dcodes, dptr, dind, out_b)
    for rep in range(3):
        out_a.fill_(-1.0)
        out_b.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_a, eager_a) and torch.equal(out_b, eager_b), f"replay {rep}"
        # eager work between replays
        assert torch.equal(q.gather_mean(dcodes, dptr, dind), eager_b)


def test_validate_option_rejects_broken_index_contracts(bf, torch):
    # option "validate": indices and list bounds are checked by a small kernel and a broken
    # contract is refused before any gather kernel is launched
    q, s, codes, dcodes = _tables(bf, torch, "uniform", 4, 100)
    N = codes.shape[0]
    q.set_option("validate", 1)
    good = torch.tensor([0, N - 1, 5], dtype=torch.int64, device="cuda")
    assert_close(q.gather_dequant(dcodes, good).cpu().numpy(),
                 orc.gather_dequant(s, codes, good.cpu().numpy()), s)
    out = torch.full((3, 100), 7.0, device="cuda")
    for bad in ([0, N, 5], [0, -1, 5]):
        with pytest.raises(bf.BifeatError) as e:
            q.gather_dequant(dcodes, torch.tensor(bad, dtype=torch.int64, device="cuda"), out)
        assert e.value.status == -1
        with pytest.raises(bf.BifeatError):
            q.gather_codes(dcodes, torch.tensor(bad, dtype=torch.int64, device="cuda"))
    assert bool((out == 7.0).all())                  # nothing was written
    ptr = torch.tensor([0, 2, 3], dtype=torch.int64, device="cuda")
    ind = torch.tensor([1, 2, 3], dtype=torch.int64, device="cuda")
    want = orc.gather_mean(s, codes, ptr.cpu().numpy(), ind.cpu().numpy())
    assert_close(q.gather_mean(dcodes, ptr, ind).cpu().numpy(), want, s)
    broken = [(torch.tensor([0, 3, 2], dtype=torch.int64, device="cuda"), ind),      # decreasing
              (torch.tensor([1, 2, 3], dtype=torch.int64, device="cuda"), ind),      # indptr[0] != 0
              (torch.tensor([0, 2, 2], dtype=torch.int64, device="cuda"), ind),      # indptr[V] != E
              (ptr, torch.tensor([1, N + 4, 3], dtype=torch.int64, device="cuda"))]  # index out of range
    for p_, i_ in broken:
        with pytest.raises(bf.BifeatError):
            q.gather_mean(dcodes, p_, i_)
        with pytest.raises(bf.BifeatError):
            q.gather_sum(dcodes, p_, i_)
    # a promised bound on the list lengths is checked as part of the contract
    q.set_option("mean_max_degree", 2)
    assert_close(q.gather_mean(dcodes, ptr, ind).cpu().numpy(), want, s)     # lists of 2 and 1
    q.set_option("mean_max_degree", 1)
    with pytest.raises(bf.BifeatError):
        q.gather_mean(dcodes, ptr, ind)
    q.set_option("mean_max_degree", 0)
    q.set_option("validate", 0)


@pytest.mark.parametrize("V", [1, 3, 17])
def test_small_requests_reach_every_codebook_slice(bf, torch, V):
    # fewer destinations / rows than column slices: every slice still gets a workgroup
    q, s, codes, dcodes = _tables(bf, torch, "vq", 8, 96, w=4, length=256)   # 24 parts, several slices
    rng = np.random.default_rng(V)
    indptr, indices = random_csr(V + 1, codes.shape[0], 6, rng)
    got = q.gather_mean(dcodes, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda())
    assert_close(got.cpu().numpy(), orc.gather_mean(s, codes, indptr, indices), s)
    idx = rng.integers(0, codes.shape[0], V).astype(np.int64)
    assert_close(q.gather_dequant(dcodes, torch.from_numpy(idx).cuda()).cpu().numpy(),
                 orc.gather_dequant(s, codes, idx), s)
