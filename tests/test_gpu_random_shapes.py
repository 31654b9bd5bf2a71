"""Seeded random configurations (shape, scheme, bit width, list lengths) through the whole
path against the oracle: the shape classes the hand-picked cases do not name."""
import os

import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk
from bifeat_inputs.device import DeviceTable
from helpers import scheme_of, assert_close, column_magnitude, REL_TOL, random_csr, gpu_build_table

pytestmark = pytest.mark.gpu

# BIFEAT_TEST_SEED=k shifts every seed below: further draws of the same distributions
SEED = 100_000 * int(os.environ.get("BIFEAT_TEST_SEED", "0"))


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


@pytest.fixture(scope="module")
def bf():
    import paper_2207_14696_amd as m
    m.load_library()
    return m


def _draw(rng):
    kind = rng.choice(["uniform", "log", "vq"], p=[0.45, 0.25, 0.3])
    D = int(rng.choice([1, 3, 4, 7, 16, 30, 64, 100, 130, 257, 512, 1000, 2304]))
    cfg = {"kind": kind, "D": D, "dtype": str(rng.choice(["f32", "f16"])), "bits": int(rng.choice([1, 2, 4, 8]))}
    if kind == "vq":
        cfg["w"] = int(rng.choice([1, 2, 3, 4, 8, 12, 16, 20, 32]))
        cfg["length"] = int(rng.choice([2, 5, 16, 64, 256, 300, 700]))
        cfg["metric"] = str(rng.choice(["l2", "cosine"]))
        if cfg["D"] > 600:                     # keeps the oracle's nearest-entry search short
            cfg["length"] = min(cfg["length"], 64)
    return cfg


@pytest.mark.parametrize("case", range(72))
def test_random_configuration(bf, torch, case):
    rng = np.random.default_rng(SEED + 1000 + case)
    c = _draw(rng)
    N = int(rng.integers(700, 2500))
    D = c["D"]
    spec = FeatureSpec(N, D, SEED + 100 + case, c["dtype"])
    x = feature_chunk(spec, 0, N).astype(np.float32)
    if c["kind"] == "uniform":
        mn, mx = orc.fit_minmax(x)
        scale, inv = orc.uniform_params(mn, mx, c["bits"])
        s = orc.Scheme.uniform(mn, scale, c["bits"])
        want_codes = orc.pack(orc.uniform_encode(x, c["bits"], mn, inv), c["bits"])
        q = bf.Quantizer(scheme_of("uniform", c["bits"]), D)
        fit = True
    elif c["kind"] == "log":
        e = orc.log_range(orc.log_fit(x))
        T, V = orc.log_tables(*e, c["bits"])
        s = orc.Scheme.log(D, V, c["bits"])
        want_codes = orc.pack(orc.log_encode(x, c["bits"], T), c["bits"])
        q = bf.Quantizer(scheme_of("log", c["bits"]), D)
        fit = True
    else:
        w, length, metric = c["w"], c["length"], c["metric"]
        cb, _ = orc.vq_train(x[:max(length, 400)], w, length, iters=2, metric=metric)
        s = orc.Scheme.vq(D, cb)
        want_codes = orc.pack(orc.vq_assign(x, w, cb, metric=metric), orc.vq_code_bits(length))
        q = bf.Quantizer(scheme_of("vq", 8, w, length, metric), D)
        q.params_set_codebooks(cb)
        fit = False
    table = DeviceTable(spec)
    codes = gpu_build_table(q, table, N, int(rng.integers(100, N + 1)), fit=fit)
    assert np.array_equal(codes.cpu().numpy(), want_codes), c

    idx = rng.integers(0, N, int(rng.integers(1, 900))).astype(np.int64)
    didx = torch.from_numpy(idx).cuda()
    assert np.array_equal(q.gather_codes(codes, didx).cpu().numpy(), want_codes[idx]), c
    assert_close(q.gather_dequant(codes, didx).cpu().numpy(), orc.gather_dequant(s, want_codes, idx), s, str(c))

    hubs = tuple(int(h) for h in rng.integers(40, 1500, int(rng.integers(0, 3))))
    V = int(rng.integers(1, 500))
    indptr, indices = random_csr(V, N, int(rng.integers(1, 40)), rng, hubs=hubs)
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    assert_close(q.gather_mean(codes, dptr, dind).cpu().numpy(), orc.gather_mean(s, want_codes, indptr, indices),
                 s, f"mean {c}")
    got = q.gather_sum(codes, dptr, dind).cpu().numpy().astype(np.float64)
    want = orc.gather_sum(s, want_codes, indptr, indices).astype(np.float64)
    n = np.maximum(np.diff(indptr), 1)[:, None]
    bound = REL_TOL * np.maximum(np.abs(want), column_magnitude(s).astype(np.float64)[None, :] * n)
    assert not (np.abs(got - want) > bound).any(), f"sum {c}"


def _build(bf, torch, c, N, seed):
    """(quantizer, oracle scheme, oracle codes, device codes) for configuration c."""
    D = c["D"]
    spec = FeatureSpec(N, D, seed, c["dtype"])
    x = feature_chunk(spec, 0, N).astype(np.float32)
    if c["kind"] == "uniform":
        mn, mx = orc.fit_minmax(x)
        scale, inv = orc.uniform_params(mn, mx, c["bits"])
        s = orc.Scheme.uniform(mn, scale, c["bits"])
        codes = orc.pack(orc.uniform_encode(x, c["bits"], mn, inv), c["bits"])
        q = bf.Quantizer(scheme_of("uniform", c["bits"]), D)
        q.params_set_uniform(mn, mx)
    elif c["kind"] == "log":
        e = orc.log_range_clipped(x, 0.02)
        T, V = orc.log_tables(*e, c["bits"])
        s = orc.Scheme.log(D, V, c["bits"])
        codes = orc.pack(orc.log_encode(x, c["bits"], T), c["bits"])
        q = bf.Quantizer(scheme_of("log", c["bits"]), D)
        q.params_set_log(*e)
    else:
        w, length, metric = c["w"], min(c["length"], 256), c["metric"]
        cb, _ = orc.vq_train(x[:max(length, 300)], w, length, iters=1, metric=metric)
        s = orc.Scheme.vq(D, cb)
        codes = orc.pack(orc.vq_assign(x, w, cb, metric=metric), orc.vq_code_bits(length))
        q = bf.Quantizer(scheme_of("vq", 8, w, length, metric), D)
        q.params_set_codebooks(cb)
    return q, s, codes, torch.from_numpy(codes).cuda()


@pytest.mark.parametrize("case", range(40))
def test_small_requests_and_fanout_bounds(bf, torch, case):
    # tiny requests (one row, one destination, a few tiles and a ragged tail) and sampled
    # blocks whose fan-out the caller states, for random configurations
    rng = np.random.default_rng(SEED + 5000 + case)
    c = _draw(rng)
    if c["D"] > 600:
        c["D"] = int(rng.choice([8, 96, 128]))
    N = int(rng.integers(300, 800))
    q, s, codes, dcodes = _build(bf, torch, c, N, 300 + case)
    for M in (1, 2, 63, 65, int(rng.integers(3, 300))):
        idx = rng.integers(0, N, M).astype(np.int64)
        got = q.gather_dequant(dcodes, torch.from_numpy(idx).cuda()).cpu().numpy()
        assert_close(got, orc.gather_dequant(s, codes, idx), s, f"dequant M={M} {c}")
    for V in (1, 2, 64, 65, int(rng.integers(3, 400))):
        f = int(rng.choice([1, 2, 5, 10, 15, 16, 17, 25, 32, 33, 64]))
        deg = rng.integers(0, f + 1, V)
        deg[rng.integers(0, V)] = f                   # the bound is attained
        indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
        indices = rng.integers(0, N, int(indptr[-1])).astype(np.int64)
        dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
        q.set_option("mean_max_degree", f)
        got = q.gather_mean(dcodes, dptr, dind).cpu().numpy()
        gsum = q.gather_sum(dcodes, dptr, dind).cpu().numpy().astype(np.float64)
        q.set_option("mean_max_degree", 0)
        assert_close(got, orc.gather_mean(s, codes, indptr, indices), s, f"mean V={V} f={f} {c}")
        want = orc.gather_sum(s, codes, indptr, indices).astype(np.float64)
        n = np.maximum(deg, 1)[:, None]
        bound = REL_TOL * np.maximum(np.abs(want), column_magnitude(s).astype(np.float64)[None, :] * n)
        assert not (np.abs(gsum - want) > bound).any(), f"sum V={V} f={f} {c}"
    # every list empty, with and without the bound
    V = int(rng.integers(1, 70))
    zptr = torch.zeros(V + 1, dtype=torch.int64, device="cuda")
    zind = torch.empty(0, dtype=torch.int64, device="cuda")
    for hint in (0, 5):
        q.set_option("mean_max_degree", hint)
        assert not q.gather_mean(dcodes, zptr, zind).any()
    q.set_option("mean_max_degree", 0)


@pytest.mark.parametrize("case", range(24))
def test_random_fits(bf, torch, case):
    # streaming fits with random chunking, special values in the table
    rng = np.random.default_rng(SEED + 9000 + case)
    D = int(rng.choice([1, 5, 32, 100, 257, 768]))
    N = int(rng.integers(200, 3000))
    dtype = str(rng.choice(["f32", "f16"]))
    spec = FeatureSpec(N, D, SEED + 900 + case, dtype)
    x = feature_chunk(spec, 0, N).astype(np.float32)
    # sprinkle zeros, NaNs and infinities (NaNs are skipped by the fits; an infinity is a
    # legitimate extreme of a column for the uniform range and ignored by the log range)
    flat = x.reshape(-1)
    k = max(1, flat.size // 200)
    flat[rng.integers(0, flat.size, k)] = 0.0
    flat[rng.integers(0, flat.size, max(1, k // 4))] = np.nan
    with_inf = case % 3 == 0
    if with_inf:
        flat[rng.integers(0, flat.size, 2)] = np.inf
    tx = torch.from_numpy(x).cuda()
    if dtype == "f16":
        tx = tx.half()
        x = tx.float().cpu().numpy()
    cuts = np.sort(rng.choice(np.arange(1, N), size=min(N - 1, int(rng.integers(0, 6))), replace=False))
    bounds = [0, *cuts.tolist(), N]

    def stream(q):
        for a, b in zip(bounds[:-1], bounds[1:]):
            q.fit_update(tx[a:b])

    bits = int(rng.choice([1, 2, 4, 8]))
    q = bf.Quantizer(scheme_of("uniform", bits), D)
    q.fit_reset()
    stream(q)
    assert q.fit_finalize() is False
    mn, mx, scale, inv = q.params_get_uniform()
    omn, omx = orc.fit_minmax(x)
    assert np.array_equal(mn, omn) and np.array_equal(mx, omx)
    # (a column whose range is infinite has scale = inf and inv = 0 on both sides)
    osc, oinv = orc.uniform_params(omn, omx, bits)
    assert np.array_equal(scale, osc) and np.array_equal(inv, oinv)

    frac = float(rng.choice([0.0, 0.001, 0.01, 0.1, 0.3]))
    ql = bf.Quantizer(scheme_of("log", bits), D)
    ql.fit_set_log_clip(frac)
    ql.fit_reset()
    again, passes = True, 0
    while again:
        stream(ql)
        again = ql.fit_finalize()
        passes += 1
    assert passes == (3 if frac > 0 else 1)
    want = orc.log_range_clipped(x, frac) if frac > 0 else orc.log_range(orc.log_fit(x))
    assert ql.params_get_log()[:2] == want
