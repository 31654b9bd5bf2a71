"""GPU tests of the call contract around the fused mean (Appendix A.1): 32-bit list
entries, the promised bound on list lengths (a broken promise must be loud, never stale
memory), table widths at the edge of the staged decode kernel's LDS, and the workspace
policy of the vector-code gathers (reserve, growth, graph capture)."""
import numpy as np
import pytest

import oracle as orc
from helpers import assert_close, random_csr, scheme_of
from test_gpu_parity import _tables

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


I32_CASES = [("uniform", 1, 768), ("uniform", 2, 128), ("uniform", 4, 100), ("uniform", 8, 128),
             ("uniform", 4, 37), ("uniform", 4, 768), ("log", 1, 64), ("log", 2, 100), ("log", 4, 128),
             ("log", 8, 200), ("log", 4, 37), ("vq", 8, 64), ("vq", 8, 23), ("vq", 8, 96)]


@pytest.mark.parametrize("kind,bits,D", I32_CASES)
def test_int32_list_entries_match_oracle(bf, torch, kind, bits, D):
    # the same block through bifeat_gather_mean_i32 / bifeat_gather_sum_i32: every kernel family
    # (short-list forms with and without the caller's bound, general kernels, vector codes)
    w = {23: 5, 96: 16}.get(D, 8)
    q, s, codes, dcodes = _tables(bf, torch, kind, bits, D, w=w)
    rng = np.random.default_rng(11)
    indptr, indices = random_csr(1203, codes.shape[0], 12, rng, hubs=(15, 17, 33, 64, 65, 300, 700))
    dptr = torch.from_numpy(indptr).cuda()
    d32 = torch.from_numpy(indices.astype(np.int32)).cuda()
    want = orc.gather_mean(s, codes, indptr, indices)
    out = torch.full((1203, D), float("nan"), device="cuda")
    q.gather_mean(dcodes, dptr, d32, out)
    assert_close(out.cpu().numpy(), want, s, "i32 mean")
    got64 = q.gather_mean(dcodes, dptr, torch.from_numpy(indices).cuda())
    assert torch.equal(out, got64)          # same kernels, same order of operations
    # sum aggregator
    wsum = orc.gather_sum(s, codes, indptr, indices)
    gsum = q.gather_sum(dcodes, dptr, d32)
    assert torch.equal(gsum, q.gather_sum(dcodes, dptr, torch.from_numpy(indices).cuda()))
    n = np.maximum(np.diff(indptr), 1)[:, None]
    from helpers import column_magnitude, REL_TOL
    bound = REL_TOL * np.maximum(np.abs(wsum.astype(np.float64)), column_magnitude(s)[None, :] * n)
    assert not (np.abs(gsum.cpu().numpy() - wsum.astype(np.float64)) > bound).any()
    # short lists with the caller's bound: one short-list kernel alone
    indptr, indices = random_csr(777, codes.shape[0], 7, rng)
    q.set_option("mean_max_degree", 7)
    out = torch.full((777, D), float("nan"), device="cuda")
    q.gather_mean(dcodes, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices.astype(np.int32)).cuda(), out)
    q.set_option("mean_max_degree", 0)
    assert_close(out.cpu().numpy(), orc.gather_mean(s, codes, indptr, indices), s, "i32 short lists")
    assert q.poll_status()


def test_int32_entries_need_a_table_that_fits(bf, torch):
    q, s, codes, dcodes = _tables(bf, torch, "uniform", 4, 100)
    ptr = torch.tensor([0, 1], dtype=torch.int64, device="cuda")
    ind = torch.tensor([3], dtype=torch.int32, device="cuda")
    lib = bf.load_library()
    rc = lib.bifeat_gather_mean_i32(q._h, dcodes.data_ptr(), 1 << 31, ptr.data_ptr(), ind.data_ptr(), 1, 1,
                                    torch.empty((1, 100), device="cuda").data_ptr(), 0)
    assert rc == bf.EINVAL
    q.set_option("validate", 1)
    with pytest.raises(bf.BifeatError) as e:
        q.gather_mean(dcodes, ptr, ind)
    assert e.value.status == bf.ENOTSUP
    q.set_option("validate", 0)


@pytest.mark.parametrize("kind,bits,D,promise,longest", [
    ("uniform", 4, 100, 10, 11), ("uniform", 4, 100, 10, 300), ("uniform", 1, 768, 15, 16),
    ("uniform", 2, 128, 5, 90), ("uniform", 8, 128, 25, 70), ("log", 1, 64, 10, 40),
    ("log", 2, 100, 15, 16), ("log", 4, 128, 10, 65), ("log", 8, 200, 25, 100),
    ("vq", 8, 64, 10, 33), ("vq", 8, 96, 25, 200)])
def test_broken_length_promise_is_reported_not_silent(bf, torch, kind, bits, D, promise, longest):
    # mean_max_degree = d promises lists of at most d entries; the kernels that rely on it
    # cover lists up to their own capacity (>= d).  A list beyond that capacity cannot be
    # averaged by them: its row must come back as NaN (never stale memory), the status word
    # must be raised, the next call must refuse, and every other row must still be right.
    w = {96: 16}.get(D, 8)
    q, s, codes, dcodes = _tables(bf, torch, kind, bits, D, w=w)
    rng = np.random.default_rng(5)
    V = 901
    indptr, indices = random_csr(V, codes.shape[0], promise, rng)
    want = orc.gather_mean(s, codes, indptr, indices)
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    q.set_option("mean_max_degree", promise)
    out = torch.full((V, D), 7.0, device="cuda")
    q.gather_mean(dcodes, dptr, dind, out)
    assert q.poll_status()                                   # promise kept: nothing raised
    assert_close(out.cpu().numpy(), want, s, "promise kept")
    # now break it: two lists of `longest` entries (first tile and a later one)
    bad = [5, 640]
    deg = np.diff(indptr)
    deg[bad] = longest
    ptr2 = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    ind2 = rng.integers(0, codes.shape[0], int(ptr2[-1])).astype(np.int64)
    want2 = orc.gather_mean(s, codes, ptr2, ind2)
    out = torch.full((V, D), 7.0, device="cuda")
    q.gather_mean(dcodes, torch.from_numpy(ptr2).cuda(), torch.from_numpy(ind2).cuda(), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ok = np.ones(V, bool)
    over = np.isnan(got).all(axis=1)
    if over.any():
        # the kernel's capacity is below `longest`: both rows NaN, everything else correct
        assert sorted(np.flatnonzero(over).tolist()) == bad
        ok[bad] = False
        with pytest.raises(bf.BifeatError) as e:             # the next call on the handle refuses
            q.gather_mean(dcodes, dptr, dind)
        assert e.value.status == bf.EINVAL
        assert q.poll_status()                               # ... and that cleared the word
    else:
        # the kernel's own capacity covered the longer lists: they are simply correct
        assert q.poll_status()
    assert not np.isnan(got[ok]).any()
    assert_close(got[ok], want2[ok], s, "rows inside the promise")
    # the explicit query reports it too (and clears it)
    q.gather_mean(dcodes, torch.from_numpy(ptr2).cuda(), torch.from_numpy(ind2).cuda(), out)
    assert q.poll_status() == (not over.any())
    assert q.poll_status()
    q.set_option("mean_max_degree", 0)
    # without the promise the same block is averaged in full
    assert_close(q.gather_mean(dcodes, torch.from_numpy(ptr2).cuda(), torch.from_numpy(ind2).cuda()).cpu().numpy(),
                 want2, s, "no promise")


def test_capacity_of_short_list_kernels_is_what_the_cases_assume(bf, torch):
    # the cases above must include lists beyond every short-list kernel's capacity
    q, s, codes, dcodes = _tables(bf, torch, "uniform", 4, 100)
    rng = np.random.default_rng(6)
    indptr, indices = random_csr(300, codes.shape[0], 10, rng, hubs=(65,))
    q.set_option("mean_max_degree", 10)
    out = q.gather_mean(dcodes, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda())
    assert not q.poll_status()
    assert torch.isnan(out[1]).all() and not torch.isnan(out[2:]).any()
    q.set_option("mean_max_degree", 0)


@pytest.mark.parametrize("D", [7680, 7684, 8192])
def test_one_bit_table_wider_than_the_staged_kernels_lds(bf, torch, D):
    # 1-bit uniform codes, D up to 8192: the packed row still fits one wavefront's loads, but
    # the staged decode kernel's parameters (2*D floats) exceed a workgroup's 64 KB of LDS
    # beyond D = 7680: those tables take the flat kernel
    from bifeat_inputs import FeatureSpec, feature_chunk
    spec = FeatureSpec(257, D, 21)
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, 1)
    s = orc.Scheme.uniform(mn, scale, 1)
    codes = orc.pack(orc.uniform_encode(x, 1, mn, inv), 1)
    q = bf.Quantizer(scheme_of("uniform", 1), D)
    q.params_set_uniform(mn, mx)
    assert q.row_bytes == codes.shape[1]
    dcodes = torch.from_numpy(codes).cuda()
    rng = np.random.default_rng(3)
    idx = rng.integers(0, spec.N, 333).astype(np.int64)
    got = q.gather_dequant(dcodes, torch.from_numpy(idx).cuda()).cpu().numpy()
    assert_close(got, orc.gather_dequant(s, codes, idx), s, f"gather_dequant D={D}")
    indptr, indices = random_csr(65, spec.N, 9, rng, hubs=(40,))
    got = q.gather_mean(dcodes, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()).cpu().numpy()
    assert_close(got, orc.gather_mean(s, codes, indptr, indices), s, f"gather_mean D={D}")


def test_vector_code_workspace_reserve_growth_and_capture(bf, torch):
    # the vector-code gathers transpose the requested rows into a library workspace.  It grows
    # with the largest request, an outgrown buffer stays valid for graphs captured earlier, and
    # nothing is allocated while a stream is capturing (a too-large request is then served by
    # the kernels that need no workspace) - results are the oracle's in every case.
    q, s, codes, dcodes = _tables(bf, torch, "vq", 8, 64)
    rng = np.random.default_rng(9)

    def block(V):
        indptr, indices = random_csr(V, codes.shape[0], 9, rng)
        return indptr, indices, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()

    small = block(300)
    out_small = torch.empty((300, 64), device="cuda")
    q.set_option("mean_max_degree", 9)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        q.gather_mean(dcodes, small[2], small[3], out_small)          # sizes the workspace
        stream.synchronize()
        g_small = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_small, stream=stream):
            q.gather_mean(dcodes, small[2], small[3], out_small)
        # a larger request inside a capture: no allocation, still the right answer on replay
        big = block(4000)
        out_big = torch.empty((4000, 64), device="cuda")
        g_big = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_big, stream=stream):
            q.gather_mean(dcodes, big[2], big[3], out_big)
    want_small = orc.gather_mean(s, codes, small[0], small[1])
    want_big = orc.gather_mean(s, codes, big[0], big[1])
    for rep in range(3):
        out_small.fill_(float("nan"))
        out_big.fill_(float("nan"))
        g_small.replay()
        g_big.replay()
        torch.cuda.synchronize()
        assert_close(out_small.cpu().numpy(), want_small, s, f"captured small, replay {rep}")
        assert_close(out_big.cpu().numpy(), want_big, s, f"captured big, replay {rep}")
        if rep == 0:
            # eager growth between replays: the small graph's workspace must stay valid
            q.reserve(100_000)
            huge = block(9000)
            got = q.gather_mean(dcodes, huge[2], huge[3])
            assert_close(got.cpu().numpy(), orc.gather_mean(s, codes, huge[0], huge[1]), s, "after growth")
    q.set_option("mean_max_degree", 0)
    assert q.poll_status()


ALIGN_CASES = [("uniform", 1, 768, 96, 128), ("uniform", 4, 100, 64, 64), ("uniform", 4, 96, 48, 64),
               ("uniform", 2, 128, 32, 32), ("uniform", 8, 200, 208, 256), ("uniform", 4, 768, 384, 384),
               ("log", 1, 768, 96, 128), ("log", 2, 300, 80, 128), ("log", 4, 160, 80, 128),
               ("vq", 8, 768, 96, 128), ("vq", 8, 64, 16, 16)]


@pytest.mark.parametrize("kind,bits,D,payload,stride", ALIGN_CASES)
def test_line_aligned_table_layout(bf, torch, kind, bits, D, payload, stride):
    # option "row_align" = 128: same codes, same decoded values and means; only the distance
    # from row to row changes, and the bytes between the codes and the next row are zero
    from bifeat_inputs import FeatureSpec, feature_chunk
    from bifeat_inputs.device import DeviceTable
    from helpers import gpu_build_table
    w, length = 8, 256 if D == 768 else 32
    q0, s, codes, _ = _tables(bf, torch, kind, bits, D, N=2003, w=w, length=length)
    assert codes.shape[1] == payload == q0.row_bytes
    q = bf.Quantizer(q0.scheme, D, row_align=128)
    assert q.row_bytes == stride
    if kind == "uniform":
        q.params_set_uniform(*q0.params_get_uniform()[:2])
    elif kind == "log":
        q.params_set_log(*q0.params_get_log()[:2])
    else:
        q.params_set_codebooks(q0.params_get_codebooks())
    table = gpu_build_table(q, DeviceTable(FeatureSpec(2003, D, 6)), 2003, 700, fit=False)
    got = table.cpu().numpy()
    assert got.shape == (2003, stride)
    assert np.array_equal(got[:, :payload], codes) and not got[:, payload:].any()
    rng = np.random.default_rng(8)
    idx = rng.integers(0, 2003, 1501).astype(np.int64)
    didx = torch.from_numpy(idx).cuda()
    assert np.array_equal(q.gather_codes(table, didx).cpu().numpy()[:, :payload], orc.gather_codes(codes, idx))
    assert_close(q.gather_dequant(table, didx).cpu().numpy(), orc.gather_dequant(s, codes, idx), s, "dequant")
    if kind != "vq":
        q.set_option("dequant_flat", 1)
        assert_close(q.gather_dequant(table, didx).cpu().numpy(), orc.gather_dequant(s, codes, idx), s, "flat")
        q.set_option("dequant_flat", 0)
    indptr, indices = random_csr(907, 2003, 11, rng, hubs=(15, 17, 40, 65, 300))
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    want = orc.gather_mean(s, codes, indptr, indices)
    assert_close(q.gather_mean(table, dptr, dind).cpu().numpy(), want, s, "mean")
    for opt in ("mean_lean", "vq_sliced"):
        q.set_option(opt, 0)
    assert_close(q.gather_mean(table, dptr, dind).cpu().numpy(), want, s, "mean, general kernels")
    for opt in ("mean_lean", "vq_sliced"):
        q.set_option(opt, 1)
    indptr, indices = random_csr(500, 2003, 9, rng)
    q.set_option("mean_max_degree", 9)
    got = q.gather_mean(table, torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda())
    assert_close(got.cpu().numpy(), orc.gather_mean(s, codes, indptr, indices), s, "mean, bounded lists")
    assert q.poll_status()
