"""The named workloads: table shape, quantization scheme, graph, fan-outs.

Shapes follow the benchmark configurations (a tiny random graph; a
products-scale graph with D=100; a Papers100M-shaped table, 111M x 128 with a
3-hop fan-out; a MAG240M-shaped fp16 table, 244M x 768; a 100M x 768 table for
the 96 x 256-entry vector-quantized form).  All data are synthetic and seeded;
they stand in for those datasets, none of which is needed or read.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

from .features import FeatureSpec
from .graphs import PowerLawGraph, UniformGraph


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    D: int
    dtype: str                  # storage dtype of the raw table
    kind: str                   # "uniform" | "log" | "vq"
    bits: int                   # scalar schemes: bits per value
    graph: str                  # "uniform" | "powerlaw"
    avg_degree: float
    fanouts: Tuple[int, ...]    # seed side outward
    batch: int
    seed_mode: str = "uniform"  # "uniform" | "degree"
    cap: int = 10_000
    vq_width: int = 8
    vq_length: int = 256
    vq_metric: str = "l2"       # "l2" | "cosine"
    log_clip: float = 0.0       # "log": fraction of the magnitudes clipped at each tail
    seed: int = 0

    @property
    def spec(self) -> FeatureSpec:
        return FeatureSpec(self.N, self.D, self.seed, self.dtype)

    def scaled(self, N: int, **kw) -> "Workload":
        """Same shape of work on a smaller table (for parity tests)."""
        return replace(self, N=N, name=f"{self.name}@{N}", **kw)


WORKLOADS = {
    "tiny": Workload("tiny", 10_000, 128, "f32", "uniform", 8, "uniform", 15, (10,), 1024),
    "mid": Workload("mid", 2_400_000, 100, "f32", "uniform", 4, "powerlaw", 15, (25, 10), 1024),
    "large": Workload("large", 111_000_000, 128, "f32", "uniform", 2, "powerlaw", 15,
                      (15, 10, 5), 1024, seed_mode="degree"),
    "largest1": Workload("largest1", 244_000_000, 768, "f16", "uniform", 1, "powerlaw", 12,
                         (25, 15), 1024),
    "largest4": Workload("largest4", 244_000_000, 768, "f16", "uniform", 4, "powerlaw", 12,
                         (25, 15), 1024),
    "vq": Workload("vq", 100_000_000, 768, "f32", "vq", 8, "powerlaw", 15, (25, 10), 4096),
    # the paper's headline scalar setting (Appendix B: 1 bit, sign only) on the "largest" table
    "log1": Workload("log1", 244_000_000, 768, "f16", "log", 1, "powerlaw", 12, (25, 15), 1024),
    # the paper's own scalar codes at 2 bits with tail clipping (Sec. 3.1, Appendix C) on the
    # "large" table and sampling
    "log2": Workload("log2", 111_000_000, 128, "f32", "log", 2, "powerlaw", 15, (15, 10, 5), 1024,
                     seed_mode="degree", log_clip=0.01),
    # the same codes at 4 bits (a sixteen-entry decode table per value: no integer-sum form)
    "log4": Workload("log4", 111_000_000, 128, "f32", "log", 4, "powerlaw", 15, (15, 10, 5), 1024,
                     seed_mode="degree", log_clip=0.01),
    # the paper's large-graph vector setting (Appendix B: width 16, length 2048, i.e.
    # two-byte indices, cosine search) on the "large" table and sampling
    "vq2k": Workload("vq2k", 111_000_000, 128, "f32", "vq", 8, "powerlaw", 15, (15, 10, 5), 1024,
                     seed_mode="degree", vq_width=16, vq_length=2048, vq_metric="cosine"),
}


def make_graph(w: Workload):
    if w.graph == "uniform":
        return UniformGraph(w.N, int(w.avg_degree), w.seed)
    return PowerLawGraph(w.N, w.avg_degree, 2.1, w.cap, w.seed)


# minibatches concatenated into one launch by default (what a prefetching
# loader hands over); 1 = a single minibatch per launch
BATCHES_PER_STEP = {"tiny": 64, "mid": 64, "large": 8, "largest1": 32, "largest4": 32, "vq": 8,
                    "vq2k": 8, "log2": 8, "log4": 8, "log1": 32}


def launch_set(w: Workload, graph, set_index: int, L: int):
    """Launch-set ``set_index``: L independently sampled minibatches with their
    per-hop CSR blocks concatenated (destinations of all minibatches one after
    the other) and their input-node lists concatenated.
    Returns (hops, inputs): hops[h] = (indptr int64 [V+1], indices int64 [E])."""
    import numpy as np
    from .graphs import draw_seeds, sample_blocks
    mbs = []
    for l in range(L):
        bi = set_index * L + l
        seeds = draw_seeds(graph, w.batch, w.seed, bi, w.seed_mode)
        mbs.append(sample_blocks(graph, seeds, w.fanouts, w.seed, bi))
    hops = []
    for h in range(len(w.fanouts)):
        ptr, off = [np.zeros(1, np.int64)], 0
        for blocks, _ in mbs:
            ptr.append(blocks[h].indptr[1:] + off)
            off += blocks[h].E
        hops.append((np.concatenate(ptr), np.concatenate([b[h].indices for b, _ in mbs])))
    return hops, np.concatenate([inp for _, inp in mbs])


def two_round_set(w: Workload, graph, set_index: int, L: int):
    """The two outermost blocks of launch-set ``set_index`` for a two-round
    aggregation: L minibatches concatenated, the outer block's lists holding
    table rows and the seed-side block's lists renumbered to positions among the
    outer block's destinations (each minibatch's frontier is sorted, so a binary
    search renumbers them).  Returns (indptr1, indices1, indptr2, indices2)."""
    import numpy as np
    from .graphs import draw_seeds, sample_blocks
    H = len(w.fanouts)
    assert H >= 2
    p1, i1, p2, i2 = [np.zeros(1, np.int64)], [], [np.zeros(1, np.int64)], []
    o1 = o2 = voff = 0
    for l in range(L):
        bi = set_index * L + l
        blocks, _ = sample_blocks(graph, draw_seeds(graph, w.batch, w.seed, bi, w.seed_mode), w.fanouts, w.seed, bi)
        outer, inner = blocks[H - 1], blocks[H - 2]
        local = np.searchsorted(outer.dst, inner.indices)
        assert np.array_equal(outer.dst[local], inner.indices)
        p1.append(outer.indptr[1:] + o1)
        i1.append(outer.indices)
        p2.append(inner.indptr[1:] + o2)
        i2.append(local + voff)
        o1 += outer.E
        o2 += inner.E
        voff += outer.V
    return tuple(np.concatenate(a).astype(np.int64) for a in (p1, i1, p2, i2))
