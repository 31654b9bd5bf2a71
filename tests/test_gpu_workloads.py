"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times (L minibatches per launch, whole blocks, every hop with the sampler's fan-out
passed as the bound on the list lengths) and, next to it, without that bound.

The tables are far too large for the oracle to sweep (up to 187 G values), so:
  * fitted per-column min/max are checked against torch.amin/amax over the same
    chunks (an independent routine), their witness rows are regenerated on the
    host (attainment) and every sampled row is checked to lie inside (bound);
    the workloads small enough (tiny, mid) also get the oracle's full fit;
  * scale / inv derived from them must equal the oracle's bit for bit;
  * for a sample of input rows, and - on every hop's block - for every destination
    of the launch's first minibatch (up to 8192), contiguous runs in the middle and
    at the end of the block and a random sample, the oracle regenerates exactly the
    table rows involved, encodes them itself, and its packed rows / decoded rows /
    means are compared with what the GPU produced from its resident table (codes
    bit-exact, floats 1e-5).
"""
import numpy as np
import pytest

import oracle as orc
from bifeat_inputs import (WORKLOADS, BATCHES_PER_STEP, make_graph, launch_set, two_round_set,
                           feature_rows, feature_chunk)
from helpers import assert_close, column_magnitude, scheme_of

pytestmark = pytest.mark.gpu

CHUNK = 1 << 20
N_DST_SAMPLE = 192
N_ROW_SAMPLE = 1024
RUN = 1024                     # contiguous destinations checked in the middle and at the end
FIRST_MINIBATCH_CAP = 8192     # destinations of the first minibatch checked (all, up to this)


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


def _stream_table(torch, w, quantizers, fit):
    """Generate the table chunk by chunk on the GPU; fit (optionally) and
    quantize with every quantizer in ``quantizers``.  Returns
    (codes per quantizer, torch min, torch max, witness rows of min / max)."""
    from bifeat_inputs.device import DeviceTable
    table = DeviceTable(w.spec)
    buf = torch.empty((min(CHUNK, w.N), w.D), dtype=table.torch_dtype, device="cuda")
    tmin = tmax = amin = amax = None
    if fit:
        for q in quantizers:
            q.fit_reset()
        for r0 in range(0, w.N, CHUNK):
            n = min(CHUNK, w.N - r0)
            x = table.chunk(r0, n, buf[:n])
            for q in quantizers:
                q.fit_update(x)
            lo, ilo = x.min(dim=0)
            hi, ihi = x.max(dim=0)
            if tmin is None:
                tmin, tmax, amin, amax = lo.clone(), hi.clone(), ilo + r0, ihi + r0
            else:
                sel = lo < tmin
                tmin, amin = torch.where(sel, lo, tmin), torch.where(sel, ilo + r0, amin)
                sel = hi > tmax
                tmax, amax = torch.where(sel, hi, tmax), torch.where(sel, ihi + r0, amax)
        for q in quantizers:
            q.fit_finalize()
    codes = [torch.empty((w.N, q.row_bytes), dtype=torch.uint8, device="cuda") for q in quantizers]
    for r0 in range(0, w.N, CHUNK):
        n = min(CHUNK, w.N - r0)
        x = table.chunk(r0, n, buf[:n])
        for q, c in zip(quantizers, codes):
            q.quantize(x, c, r0)
    torch.cuda.synchronize()
    del buf
    if fit:
        return codes, tmin.float().cpu().numpy(), tmax.float().cpu().numpy(), \
            amin.cpu().numpy(), amax.cpu().numpy()
    return codes, None, None, None, None


def _check_uniform_params(w, q, tmin, tmax, amin, amax):
    mn, mx, scale, inv = q.params_get_uniform()
    tmin = np.where(tmin == 0, np.float32(0), tmin)
    tmax = np.where(tmax == 0, np.float32(0), tmax)
    assert np.array_equal(mn, tmin) and np.array_equal(mx, tmax)
    # attainment: the witness rows, regenerated on the host, hold min / max
    cols = np.arange(w.D)
    assert np.array_equal(feature_rows(w.spec, amin).astype(np.float32)[cols, cols], mn)
    assert np.array_equal(feature_rows(w.spec, amax).astype(np.float32)[cols, cols], mx)
    oscale, oinv = orc.uniform_params(mn, mx, w.bits)
    assert np.array_equal(scale.view(np.uint32), oscale.view(np.uint32))
    assert np.array_equal(inv.view(np.uint32), oinv.view(np.uint32))
    if w.N * w.D <= 300_000_000:      # the oracle can sweep this one whole
        omn = omx = None
        for r0 in range(0, w.N, 400_000):
            omn, omx = orc.fit_minmax(feature_chunk(w.spec, r0, min(400_000, w.N - r0)), omn, omx)
        assert np.array_equal(omn, mn) and np.array_equal(omx, mx)
    return mn, mx, scale, inv


def _oracle_rows(w, rows, encode):
    """Packed oracle sub-table for the sorted unique row ids ``rows``."""
    x = feature_rows(w.spec, rows).astype(np.float32)
    return x, encode(x)


def _dst_sample(w, g, h, indptr, rng):
    """Destinations of hop h whose rows are compared: every destination of the launch-set's
    first minibatch (a whole minibatch as one launch serves it), contiguous runs in the
    middle and at the very end (tile tails, the last workgroup), the extremes of the list
    lengths, and a random sample."""
    from bifeat_inputs import draw_seeds, sample_blocks
    V = indptr.shape[0] - 1
    deg = np.diff(indptr)
    first = sample_blocks(g, draw_seeds(g, w.batch, w.seed, 0, w.seed_mode), w.fanouts, w.seed, 0)[0][h].V
    first = min(first, V, FIRST_MINIBATCH_CAP)
    run = min(RUN, V)
    dst = np.concatenate([np.arange(first), np.arange(V // 2, min(V, V // 2 + run)), np.arange(V - run, V),
                          rng.choice(V, size=min(N_DST_SAMPLE, V), replace=False),
                          [int(deg.argmax()), int(deg.argmin())]])
    return np.unique(dst)


def _run_iteration_checks(torch, w, q, codes, s_of, encode, bound=None):
    """The per-iteration calls as bench.py launches them - L minibatches per launch, and every
    hop both with the sampler's fan-out passed as the bound on the list lengths (bench.py's
    default: one short-list kernel per hop) and without it (the two- and three-kernel
    launch sets) - checked against the oracle on sampled rows and destinations."""
    g = make_graph(w)
    L = BATCHES_PER_STEP[w.name]
    hops, inputs = launch_set(w, g, 0, L)
    rng = np.random.default_rng(0)
    d_inputs = torch.from_numpy(inputs).cuda()
    feats = q.gather_dequant(codes, d_inputs)
    rows_codes = q.gather_codes(codes, d_inputs)
    d_hops = [(torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()) for indptr, indices in hops]
    outs = {}
    for hinted in (True, False):
        for h, (dp, di) in enumerate(d_hops):
            q.set_option("mean_max_degree", w.fanouts[h] if hinted else 0)
            outs[hinted, h] = q.gather_mean(codes, dp, di)
        q.set_option("mean_max_degree", 0)
        assert q.poll_status()          # the sampler keeps its promise: nothing raised
    # 32-bit list entries on the outermost hop, as a loader with a table below 2^31 rows passes them
    outer = len(hops) - 1
    q.set_option("mean_max_degree", w.fanouts[outer])
    out32 = q.gather_mean(codes, d_hops[outer][0], d_hops[outer][1].to(torch.int32))
    q.set_option("mean_max_degree", 0)
    assert torch.equal(out32, outs[True, outer])
    del out32
    torch.cuda.synchronize()

    # ---- sampled input rows: packed bytes bit-exact, decoded rows within tolerance
    pick = np.sort(rng.choice(inputs.shape[0], size=min(N_ROW_SAMPLE, inputs.shape[0]), replace=False))
    uniq, inv_map = np.unique(inputs[pick], return_inverse=True)
    x, ocodes = _oracle_rows(w, uniq, encode)
    if bound is not None:
        assert np.all(x >= bound[0][None, :]) and np.all(x <= bound[1][None, :])
    s = s_of()
    dpick = torch.from_numpy(pick).cuda()
    assert np.array_equal(rows_codes[dpick].cpu().numpy(), ocodes[inv_map])
    assert_close(feats[dpick].cpu().numpy(), orc.gather_dequant(s, ocodes, inv_map), s,
                 f"{w.name} gather_dequant")

    # ---- destinations of every hop's block
    for h, (indptr, indices) in enumerate(hops):
        dst = _dst_sample(w, g, h, indptr, rng)
        lists = [indices[indptr[v]:indptr[v + 1]] for v in dst]
        cat = np.concatenate(lists)
        uniq = np.unique(cat)
        x, ocodes = _oracle_rows(w, uniq, encode)
        sub_ptr = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int64)
        sub_idx = np.searchsorted(uniq, cat).astype(np.int64)
        want = orc.gather_mean(s, ocodes, sub_ptr, sub_idx)
        ddst = torch.from_numpy(dst).cuda()
        for hinted in (True, False):
            got = outs[hinted, h][ddst].cpu().numpy()
            assert_close(got, want, s, f"{w.name} gather_mean hop {h} "
                                       f"{'with' if hinted else 'without'} the fan-out bound")
        # the two launch sets must also agree with each other on every destination
        a, b = outs[True, h], outs[False, h]
        A = torch.from_numpy(column_magnitude(s).astype(np.float32)).cuda()[None, :]
        assert bool(((a - b).abs() <= 2e-5 * torch.maximum(a.abs(), A)).all()), f"{w.name} hop {h}: launch sets differ"


def _run_two_round_checks(torch, w, q, codes, s_of, encode):
    """bifeat_gather_mean_2hop over the two outermost blocks of the launch-set, as bench.py's
    two-round leg calls it (the larger fan-out passed as the bound) and without the bound:
    sampled seeds against the oracle, which regenerates and encodes exactly the rows involved."""
    if len(w.fanouts) < 2:
        return
    g = make_graph(w)
    L = BATCHES_PER_STEP[w.name]
    p1, i1, p2, i2 = two_round_set(w, g, 0, L)
    cu = lambda a: torch.from_numpy(a).cuda()
    dp1, di1, dp2, di2 = cu(p1), cu(i1), cu(p2), cu(i2)
    H = len(w.fanouts)
    outs = {}
    for hinted in (True, False):
        q.set_option("mean_max_degree", max(w.fanouts[H - 1], w.fanouts[H - 2]) if hinted else 0)
        outs[hinted] = q.gather_mean_2hop(codes, dp1, di1, dp2, di2)
        q.set_option("mean_max_degree", 0)
        assert q.poll_status()
    rng = np.random.default_rng(1)
    V2 = p2.shape[0] - 1
    run = min(RUN, V2)
    deg2 = np.diff(p2)
    dst = np.unique(np.concatenate([np.arange(min(w.batch, V2)), np.arange(V2 - run, V2),
                                    rng.choice(V2, size=min(N_DST_SAMPLE, V2), replace=False),
                                    [int(deg2.argmax()), int(deg2.argmin())]]))
    # compact copy of what those seeds touch: their lists, the outer lists they name, the rows
    lists2 = [i2[p2[v]:p2[v + 1]] for v in dst]
    us = np.unique(np.concatenate(lists2))
    lists1 = [i1[p1[u]:p1[u + 1]] for u in us]
    rows = np.unique(np.concatenate(lists1))
    _, ocodes = _oracle_rows(w, rows, encode)
    sp1 = np.concatenate([[0], np.cumsum([len(l) for l in lists1])]).astype(np.int64)
    si1 = np.searchsorted(rows, np.concatenate(lists1)).astype(np.int64)
    sp2 = np.concatenate([[0], np.cumsum([len(l) for l in lists2])]).astype(np.int64)
    si2 = np.searchsorted(us, np.concatenate(lists2)).astype(np.int64)
    s = s_of()
    want = orc.gather_mean_2hop(s, ocodes, sp1, si1, sp2, si2)
    ddst = cu(dst)
    for hinted in (True, False):
        assert_close(outs[hinted][ddst].cpu().numpy(), want, s,
                     f"{w.name} two rounds {'with' if hinted else 'without'} the bound")
    A = torch.from_numpy(column_magnitude(s).astype(np.float32)).cuda()[None, :]
    a, b = outs[True], outs[False]
    assert bool(((a - b).abs() <= 2e-5 * torch.maximum(a.abs(), A)).all()), f"{w.name}: the two kernels differ"


def _uniform_case(torch, bf, names):
    ws = [WORKLOADS[n] for n in names]
    qs = [bf.Quantizer(scheme_of("uniform", w.bits), w.D) for w in ws]
    codes, tmin, tmax, amin, amax = _stream_table(torch, ws[0], qs, fit=True)
    for w, q, c in zip(ws, qs, codes):
        mn, mx, scale, inv = _check_uniform_params(w, q, tmin, tmax, amin, amax)
        _run_iteration_checks(
            torch, w, q, c,
            s_of=lambda: orc.Scheme.uniform(mn, scale, w.bits),
            encode=lambda x: orc.pack(orc.uniform_encode(x, w.bits, mn, inv), w.bits),
            bound=(mn, mx))
        _run_two_round_checks(
            torch, w, q, c,
            s_of=lambda: orc.Scheme.uniform(mn, scale, w.bits),
            encode=lambda x: orc.pack(orc.uniform_encode(x, w.bits, mn, inv), w.bits))
    del codes
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def bf():
    import paper_2207_14696_amd as m
    m.load_library()
    return m


def test_tiny_8bit(torch, bf):
    _uniform_case(torch, bf, ["tiny"])


def test_mid_4bit(torch, bf):
    _uniform_case(torch, bf, ["mid"])


@pytest.mark.timeout(600)
def test_large_2bit(torch, bf):
    _uniform_case(torch, bf, ["large"])


@pytest.mark.timeout(900)
def test_largest_1bit_and_4bit(torch, bf):
    # one table, two packed forms built from the same two generation passes
    _uniform_case(torch, bf, ["largest1", "largest4"])


@pytest.mark.timeout(900)
def test_vq_96x256(torch, bf):
    w = WORKLOADS["vq"]
    # codebooks: the oracle's 10-round Lloyd k-means on a seeded uniform row sample
    from bifeat_inputs.features import mix64, stream_key, STREAM_MISC
    ids = (mix64(stream_key(w.seed, STREAM_MISC) + np.arange(4096, dtype=np.uint64))
           % np.uint64(w.N)).astype(np.int64)
    cb, dist = orc.vq_train(feature_rows(w.spec, ids).astype(np.float32), w.vq_width, w.vq_length, 10)
    assert np.all(np.diff(dist) <= 1e-9 * dist[0])
    q = bf.Quantizer(scheme_of("vq", 8, w.vq_width, w.vq_length), w.D)
    q.params_set_codebooks(cb)
    (codes,), *_ = _stream_table(torch, w, [q], fit=False)
    _run_iteration_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.vq(w.D, cb),
        encode=lambda x: orc.pack(orc.vq_assign(x, w.vq_width, cb), 8))
    _run_two_round_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.vq(w.D, cb),
        encode=lambda x: orc.pack(orc.vq_assign(x, w.vq_width, cb), 8))
    del codes
    torch.cuda.empty_cache()


@pytest.mark.timeout(900)
def test_vq_16x2048_cosine_two_byte(torch, bf):
    # the vector setting the paper reports for its large graphs (Appendix B): width 16,
    # 2048 entries (two-byte indices), cosine search
    w = WORKLOADS["vq2k"]
    from bifeat_inputs.features import mix64, stream_key, STREAM_MISC
    ids = (mix64(stream_key(w.seed, STREAM_MISC) + np.arange(8192, dtype=np.uint64))
           % np.uint64(w.N)).astype(np.int64)
    cb, _ = orc.vq_train(feature_rows(w.spec, ids).astype(np.float32), w.vq_width, w.vq_length, 4,
                         metric=w.vq_metric)
    q = bf.Quantizer(scheme_of("vq", 8, w.vq_width, w.vq_length, w.vq_metric), w.D)
    assert q.row_bytes == 16
    q.params_set_codebooks(cb)
    (codes,), *_ = _stream_table(torch, w, [q], fit=False)
    _run_iteration_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.vq(w.D, cb),
        encode=lambda x: orc.pack(orc.vq_assign(x, w.vq_width, cb, metric=w.vq_metric), 16))
    _run_two_round_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.vq(w.D, cb),
        encode=lambda x: orc.pack(orc.vq_assign(x, w.vq_width, cb, metric=w.vq_metric), 16))
    del codes
    torch.cuda.empty_cache()


@pytest.mark.timeout(900)
def test_log_2bit_clipped(torch, bf):
    # The paper's own scalar codes at 2 bits, range clipped at both tails (Sec. 3.1,
    # Appendix C).  The oracle cannot sort 14 G magnitudes, so the fitted range is pinned
    # by the defining property of an order statistic, counted with library reductions:
    # #{m < value} <= rank < #{m <= value}.
    from bifeat_inputs.device import DeviceTable
    w = WORKLOADS["log2"]
    q = bf.Quantizer(scheme_of("log", w.bits), w.D)
    q.fit_set_log_clip(w.log_clip)
    table = DeviceTable(w.spec)
    buf = torch.empty((CHUNK, w.D), dtype=table.torch_dtype, device="cuda")
    q.fit_reset()
    passes, again = 0, True
    while again:
        for r0 in range(0, w.N, CHUNK):
            n = min(CHUNK, w.N - r0)
            q.fit_update(table.chunk(r0, n, buf[:n]))
        again = q.fit_finalize()
        passes += 1
    assert passes == 3
    e_min, e_max, T, V = q.params_get_log()
    lo, hi = np.float32(2.0 ** e_min), np.float32(2.0 ** e_max)
    assert np.log2(np.float64(lo)) == e_min and np.log2(np.float64(hi)) == e_max
    cnt = np.zeros(5, dtype=np.int64)        # n, <lo, <=lo, <hi, <=hi
    for r0 in range(0, w.N, CHUNK):
        n = min(CHUNK, w.N - r0)
        m = table.chunk(r0, n, buf[:n]).abs()
        ok = torch.isfinite(m) & (m > 0)
        cnt += np.array([int(ok.sum()), int((ok & (m < float(lo))).sum()), int((ok & (m <= float(lo))).sum()),
                         int((ok & (m < float(hi))).sum()), int((ok & (m <= float(hi))).sum())])
    k_lo = int(np.floor(w.log_clip * (cnt[0] - 1)))
    k_hi = int(np.ceil((1.0 - w.log_clip) * (cnt[0] - 1)))
    assert cnt[1] <= k_lo < cnt[2] and cnt[3] <= k_hi < cnt[4]
    oT, oV = orc.log_tables(e_min, e_max, w.bits)
    assert np.array_equal(T, oT) and np.array_equal(V, oV)
    del buf
    (codes,), *_ = _stream_table(torch, w, [q], fit=False)
    _run_iteration_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.log(w.D, oV, w.bits),
        encode=lambda x: orc.pack(orc.log_encode(x, w.bits, oT), w.bits))
    _run_two_round_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.log(w.D, oV, w.bits),
        encode=lambda x: orc.pack(orc.log_encode(x, w.bits, oT), w.bits))
    del codes
    torch.cuda.empty_cache()


@pytest.mark.timeout(900)
def test_log_1bit(torch, bf):
    # the paper's headline scalar setting (Sec. 3.1: one bit, the sign; Appendix C calls it
    # practical for most cases) on the largest table: the streaming fit of the extreme
    # magnitudes is checked against a library reduction over the same chunks
    from bifeat_inputs.device import DeviceTable
    w = WORKLOADS["log1"]
    q = bf.Quantizer(scheme_of("log", w.bits), w.D)
    table = DeviceTable(w.spec)
    buf = torch.empty((CHUNK, w.D), dtype=table.torch_dtype, device="cuda")
    q.fit_reset()
    lo, hi = np.inf, 0.0
    for r0 in range(0, w.N, CHUNK):
        n = min(CHUNK, w.N - r0)
        x = table.chunk(r0, n, buf[:n])
        q.fit_update(x)
        m = x.abs().float()
        hi = max(hi, float(m.max()))
        lo = min(lo, float(torch.where(m > 0, m, torch.full_like(m, float("inf"))).min()))
    assert q.fit_finalize() is False
    e_min, e_max, T, V = q.params_get_log()
    assert (e_min, e_max) == orc.log_range(np.array([lo, hi], dtype=np.float32))
    oT, oV = orc.log_tables(e_min, e_max, w.bits)
    assert len(T) == 0 and np.array_equal(V, oV)
    del buf
    (codes,), *_ = _stream_table(torch, w, [q], fit=False)
    _run_iteration_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.log(w.D, oV, w.bits),
        encode=lambda x: orc.pack(orc.log_encode(x, w.bits, oT), w.bits))
    _run_two_round_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.log(w.D, oV, w.bits),
        encode=lambda x: orc.pack(orc.log_encode(x, w.bits, oT), w.bits))
    del codes
    torch.cuda.empty_cache()


@pytest.mark.timeout(900)
def test_log_4bit(torch, bf):
    # the same codes at 4 bits: a sixteen-entry decode table, the look-up mean kernel.  The
    # range is taken from a sample of the table (any range serves the parity of codes,
    # decoded rows and means; the clipped fit itself is pinned by the 2-bit workload)
    w = WORKLOADS["log4"]
    e_min, e_max = orc.log_range_clipped(feature_chunk(w.spec, 0, 200_000).astype(np.float32), w.log_clip)
    q = bf.Quantizer(scheme_of("log", w.bits), w.D)
    q.params_set_log(e_min, e_max)
    oT, oV = orc.log_tables(e_min, e_max, w.bits)
    _, _, T, V = q.params_get_log()
    assert np.array_equal(T, oT) and np.array_equal(V, oV)
    (codes,), *_ = _stream_table(torch, w, [q], fit=False)
    _run_iteration_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.log(w.D, oV, w.bits),
        encode=lambda x: orc.pack(orc.log_encode(x, w.bits, oT), w.bits))
    _run_two_round_checks(
        torch, w, q, codes,
        s_of=lambda: orc.Scheme.log(w.D, oV, w.bits),
        encode=lambda x: orc.pack(orc.log_encode(x, w.bits, oT), w.bits))
    del codes
    torch.cuda.empty_cache()
