"""Shared helpers for the GPU parity tests (not collected by pytest)."""
from __future__ import annotations

import numpy as np

import oracle as orc
from bifeat_inputs import FeatureSpec, feature_chunk, feature_rows

REL_TOL = 1e-5   # |gpu - oracle| <= REL_TOL * max(|oracle|, A_j)


def scheme_of(kind: str, bits: int, w: int = 0, length: int = 0, metric: str = "l2"):
    import paper_2207_14696_amd as bf
    k = {"uniform": bf.UNIFORM, "log": bf.LOG, "vq": bf.VQ}[kind]
    return bf.Scheme(k, bits, w, length, {"l2": bf.VQ_L2, "cosine": bf.VQ_COSINE}[metric])


def gpu_build_table(q, table, N: int, chunk_rows: int, fit: bool = True):
    """Stream the synthetic table through fit (optional) and quantize; returns
    the packed uint8 CUDA tensor [N, row_bytes]."""
    import torch
    codes = torch.empty((N, q.row_bytes), dtype=torch.uint8, device="cuda")
    buf = None
    if fit:
        q.fit_reset()
        for r0 in range(0, N, chunk_rows):
            n = min(chunk_rows, N - r0)
            buf = table.chunk(r0, n)
            q.fit_update(buf)
        q.fit_finalize()
    for r0 in range(0, N, chunk_rows):
        n = min(chunk_rows, N - r0)
        buf = table.chunk(r0, n)
        q.quantize(buf, codes, r0)
    torch.cuda.synchronize()
    return codes


def column_magnitude(s: orc.Scheme) -> np.ndarray:
    """A_j: largest decodable magnitude per column."""
    if s.kind == orc.UNIFORM:
        L = (1 << s.bits) - 1
        hi = s.a.astype(np.float64) + L * s.b.astype(np.float64)
        return np.maximum(np.abs(s.a), np.abs(hi))
    if s.kind == orc.LOG:
        return np.full(s.D, np.abs(s.a).max())
    P, length, w = s.cb.shape
    return np.abs(s.cb).max(axis=1).reshape(P * w)[:s.D]


def assert_close(got: np.ndarray, want: np.ndarray, s: orc.Scheme, what: str = ""):
    A = column_magnitude(s).astype(np.float64)[None, :]
    bound = REL_TOL * np.maximum(np.abs(want.astype(np.float64)), A)
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    bad = err > bound
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} outside 1e-5 relative; worst "
                           f"err/bound = {(err / np.maximum(bound, 1e-300)).max():.3g}")


def random_csr(V: int, N: int, max_deg: int, rng, hubs=()):
    """CSR block with empty lists, repeats and (optionally) a few long lists."""
    deg = rng.integers(0, max_deg + 1, V)
    if V > 0:
        deg[0] = 0
    for i, h in enumerate(hubs):
        if 1 + i < V:
            deg[1 + i] = h
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    indices = rng.integers(0, N, int(indptr[-1])).astype(np.int64)
    if V > 3 and deg[3] >= 2:
        indices[indptr[3] + 1] = indices[indptr[3]]
    return indptr, indices


def oracle_uniform_table(spec: FeatureSpec, bits: int):
    x = feature_chunk(spec, 0, spec.N).astype(np.float32)
    mn, mx = orc.fit_minmax(x)
    scale, inv = orc.uniform_params(mn, mx, bits)
    codes = orc.pack(orc.uniform_encode(x, bits, mn, inv), bits)
    return x, (mn, mx, scale, inv), orc.Scheme.uniform(mn, scale, bits), codes
