"""bifeat_gather_dequant_static - the entry point for callers that cannot allocate device
memory - against bifeat_gather_dequant (and the oracle), through the C ABI: two calls in a
row on the library's fixed per-GPU workspace, the second smaller than the first."""
import numpy as np
import pytest

import oracle as orc
from helpers import assert_close
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


def _static(bf, torch, q, dcodes, didx, out):
    """The raw C call: handle, table, N, idx, M, out, stream."""
    rc = bf.load_library().bifeat_gather_dequant_static(
        q._h, dcodes.data_ptr(), dcodes.shape[0], didx.data_ptr(), didx.shape[0], out.data_ptr(),
        torch.cuda.current_stream().cuda_stream)
    return rc


@pytest.mark.parametrize("kind,bits,D,w,length", [("vq", 8, 768, 8, 256), ("vq", 8, 64, 8, 32),
                                                  ("uniform", 4, 100, 0, 0), ("log", 2, 128, 0, 0)])
def test_static_workspace_matches_allocating_entry_point(bf, torch, kind, bits, D, w, length):
    q, s, codes, dcodes = _tables(bf, torch, kind, bits, D, N=3001, w=w or 8, length=length or 32)
    rng = np.random.default_rng(4)
    # a larger call first, then a smaller one: the workspace keeps the first call's contents
    for M in (5003, 1234, 1):
        idx = rng.integers(0, codes.shape[0], M).astype(np.int64)
        idx[0] = codes.shape[0] - 1
        didx = torch.from_numpy(idx).cuda()
        want = q.gather_dequant(dcodes, didx)                      # the existing entry point
        out = torch.full((M, D), float("nan"), device="cuda")
        assert _static(bf, torch, q, dcodes, didx, out) == bf.OK
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"M={M}: differs from bifeat_gather_dequant"
        assert_close(out.cpu().numpy(), orc.gather_dequant(s, codes, idx), s, f"static M={M}")
    # M = 0 is a no-op
    empty = torch.empty(0, dtype=torch.int64, device="cuda")
    assert _static(bf, torch, q, dcodes, empty, torch.empty((0, D), device="cuda")) == bf.OK


def test_static_workspace_limit_and_argument_errors(bf, torch):
    q, s, codes, dcodes = _tables(bf, torch, "vq", 8, 64, N=1001)
    lib = bf.load_library()
    # 16-byte rows: the 32 MiB array holds about 2.09 M requests; one more tile is refused
    # before anything is launched (the output pointer is never touched)
    M_ok, M_big = (32 << 20) // 16 - 32, (32 << 20) // 16
    idx = torch.zeros(M_big, dtype=torch.int64, device="cuda")
    out = torch.empty((16, 64), device="cuda")
    assert lib.bifeat_gather_dequant_static(q._h, dcodes.data_ptr(), 1001, idx.data_ptr(), M_big,
                                            out.data_ptr(), 0) == bf.ELIMIT
    assert b"static" in lib.bifeat_strerror(bf.ELIMIT)
    big_out = torch.empty((M_ok, 64), device="cuda")
    assert lib.bifeat_gather_dequant_static(q._h, dcodes.data_ptr(), 1001, idx.data_ptr(), M_ok,
                                            big_out.data_ptr(), 0) == bf.OK
    torch.cuda.synchronize()
    row0 = orc.gather_dequant(s, codes, np.zeros(1, np.int64))
    assert_close(big_out[-1:].cpu().numpy(), row0, s, "largest request, last row")
    assert_close(big_out[:1].cpu().numpy(), row0, s, "largest request, first row")
    # not fitted / validate on / null pointers
    q2 = bf.Quantizer(bf.Scheme(bf.VQ, 8, 8, 32), 64)
    assert lib.bifeat_gather_dequant_static(q2._h, dcodes.data_ptr(), 1001, idx.data_ptr(), 4,
                                            out.data_ptr(), 0) == bf.ENOTFIT
    assert lib.bifeat_gather_dequant_static(q._h, None, 1001, idx.data_ptr(), 4, out.data_ptr(), 0) == bf.EINVAL
    q.set_option("validate", 1)
    assert lib.bifeat_gather_dequant_static(q._h, dcodes.data_ptr(), 1001, idx.data_ptr(), 4,
                                            out.data_ptr(), 0) == bf.ENOTSUP
    q.set_option("validate", 0)
