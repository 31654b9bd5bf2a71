"""Seeded synthetic graphs and a fan-out neighbour sampler (host side, numpy).

Graphs are *implicit*: the degree of a node and its k-th out-neighbour are pure
functions of (seed, node, k), so a graph with billions of edges never has to be
materialised; the sampler only ever expands the nodes of a minibatch frontier.

* ``UniformGraph``: every node has the same out-degree, neighbours uniform.
* ``PowerLawGraph``: degrees follow a (shifted, capped) power law with tail
  exponent ``alpha`` and neighbours are drawn in proportion to degree
  (preferential-attachment endpoints), so rows of hub nodes are read far more
  often than the rest - the skewed access pattern of real minibatch training.

Sampling follows the usual minibatch convention: per hop, each frontier node
keeps all neighbours if it has at most ``fanout`` of them and otherwise
``fanout`` distinct neighbour slots; the next frontier is the union of the
current one and the sampled neighbours.  Distinct slots of the implicit
multigraph may name the same node; such repeats are kept (they count with
multiplicity in a mean).
"""
from __future__ import annotations

from dataclasses import dataclass
from math import gcd
from typing import List, Sequence

import numpy as np

from .features import (mix64, stream_key, STREAM_GRAPH_NBR, STREAM_SEEDS,
                       STREAM_SLOTS)

_SLOT_STRIDE = np.uint64(1 << 20)      # max degree (cap) is below this
_U53 = 2.0 ** -53


def _unit(h: np.ndarray) -> np.ndarray:
    """64-bit hash -> double in [0, 1)."""
    return (h >> np.uint64(11)).astype(np.float64) * _U53


@dataclass
class Block:
    """One hop of a sampled minibatch: for destination v (global id
    ``dst[v]``) the sampled neighbours are ``indices[indptr[v]:indptr[v+1]]``
    (global node ids)."""
    dst: np.ndarray
    indptr: np.ndarray
    indices: np.ndarray

    @property
    def V(self) -> int:
        return int(self.dst.shape[0])

    @property
    def E(self) -> int:
        return int(self.indices.shape[0])


class UniformGraph:
    def __init__(self, N: int, out_degree: int, seed: int = 0):
        self.N, self.out_degree, self.seed = int(N), int(out_degree), int(seed)
        self._key = stream_key(seed, STREAM_GRAPH_NBR)

    def degree(self, u: np.ndarray) -> np.ndarray:
        return np.full(np.shape(u), self.out_degree, dtype=np.int64)

    def neighbor(self, u: np.ndarray, slot: np.ndarray) -> np.ndarray:
        c = u.astype(np.uint64) * _SLOT_STRIDE + slot.astype(np.uint64)
        return (mix64(self._key + c) % np.uint64(self.N)).astype(np.int64)

    def node_by_mass(self, U: np.ndarray) -> np.ndarray:
        return np.minimum((U * self.N).astype(np.int64), self.N - 1)


class PowerLawGraph:
    """deg(rank) = clip(floor(d_min * ((rank + 0.5)/N)^(-1/(alpha-1))), 1, cap):
    the inverse-CDF form of a Pareto tail with exponent ``alpha``; ``d_min`` is
    solved so that the mean degree is ``avg_degree``.  Ranks are scattered over
    node ids by an affine bijection so that hubs are not adjacent in memory."""

    def __init__(self, N: int, avg_degree: float, alpha: float = 2.1,
                 cap: int = 10_000, seed: int = 0):
        assert cap < int(_SLOT_STRIDE)
        self.N, self.alpha, self.cap, self.seed = int(N), float(alpha), int(cap), int(seed)
        self.beta = 1.0 / (alpha - 1.0)
        self._key = stream_key(seed, STREAM_GRAPH_NBR)
        # affine bijection rank <-> node id
        A = int(0.6180339887 * N) | 1
        while gcd(A, N) != 1:
            A += 2
        self._A, self._B = A % N, int(0.3141592653 * N) % N
        self._Ainv = pow(self._A, -1, N) if N > 1 else 0
        # solve d_min for the requested mean degree (monotone -> bisection)
        t = (np.arange(1 << 20, dtype=np.float64) + 0.5) / float(1 << 20)
        lo, hi = 1e-3, float(cap)
        for _ in range(80):
            mid = 0.5 * (lo + hi)
            m = np.clip(np.floor(mid * t ** (-self.beta)), 1, cap).mean()
            lo, hi = (mid, hi) if m < avg_degree else (lo, mid)
        self.d_min = 0.5 * (lo + hi)
        # continuous degree-mass CDF over t = rank/N (capped part is linear)
        b = self.beta
        self._tc = min(1.0, (self.d_min / cap) ** (1.0 / b))
        self._mass_c = cap * self._tc
        self._mass_total = self._mass_c + self.d_min * (1.0 - self._tc ** (1.0 - b)) / (1.0 - b)

    # -- bijection
    def _rank(self, u: np.ndarray) -> np.ndarray:
        return (np.uint64(self._A) * u.astype(np.uint64) + np.uint64(self._B)) % np.uint64(self.N)

    def _node(self, r: np.ndarray) -> np.ndarray:
        d = (r.astype(np.uint64) + np.uint64(self.N - self._B)) % np.uint64(self.N)
        return ((np.uint64(self._Ainv) * d) % np.uint64(self.N)).astype(np.int64)

    def degree(self, u: np.ndarray) -> np.ndarray:
        t = (self._rank(np.asarray(u)).astype(np.float64) + 0.5) / self.N
        return np.clip(np.floor(self.d_min * t ** (-self.beta)), 1, self.cap).astype(np.int64)

    def node_by_mass(self, U: np.ndarray) -> np.ndarray:
        """Node drawn in proportion to degree, from a uniform U in [0,1)."""
        b = self.beta
        m = U * self._mass_total
        t_lin = m / self.cap
        inner = np.maximum(m - self._mass_c, 0.0) * (1.0 - b) / self.d_min + self._tc ** (1.0 - b)
        t_pow = inner ** (1.0 / (1.0 - b))
        t = np.where(m <= self._mass_c, t_lin, t_pow)
        r = np.minimum((t * self.N).astype(np.int64), self.N - 1)
        return self._node(r)

    def neighbor(self, u: np.ndarray, slot: np.ndarray) -> np.ndarray:
        c = u.astype(np.uint64) * _SLOT_STRIDE + slot.astype(np.uint64)
        return self.node_by_mass(_unit(mix64(self._key + c)))


def draw_seeds(graph, count: int, seed: int, batch: int, mode: str = "uniform") -> np.ndarray:
    """``count`` distinct seed nodes of minibatch ``batch``: uniform over node
    ids, or in proportion to degree (``mode='degree'``)."""
    key = stream_key(seed, STREAM_SEEDS)
    count = min(count, graph.N)
    got = np.empty(0, dtype=np.int64)
    rnd = 0
    while got.shape[0] < count:
        n = 2 * count
        c = (np.uint64(batch) << np.uint64(40)) + (np.uint64(rnd) << np.uint64(32)) \
            + np.arange(n, dtype=np.uint64)
        h = mix64(key + c)
        cand = (h % np.uint64(graph.N)).astype(np.int64) if mode == "uniform" \
            else graph.node_by_mass(_unit(h))
        allc = np.concatenate([got, cand])
        _, first = np.unique(allc, return_index=True)
        got = allc[np.sort(first)]
        rnd += 1
    return got[:count]


def sample_blocks(graph, seeds: np.ndarray, fanouts: Sequence[int], seed: int,
                  batch: int):
    """Fan-out sampling, seed side outward (``fanouts[0]`` applies at the
    seeds).  Returns (blocks, input_nodes): ``blocks[h]`` has the frontier
    after h hops as destinations; ``input_nodes`` is the final frontier, the
    rows whose features the minibatch needs."""
    key = stream_key(seed, STREAM_SLOTS)
    frontier = np.unique(np.asarray(seeds, dtype=np.int64))
    blocks: List[Block] = []
    for hop, f in enumerate(fanouts):
        dst = frontier
        deg = graph.degree(dst)
        n = np.minimum(deg, f)
        indptr = np.zeros(dst.shape[0] + 1, dtype=np.int64)
        np.cumsum(n, out=indptr[1:])
        E = int(indptr[-1])
        owner = np.repeat(np.arange(dst.shape[0], dtype=np.int64), n)
        k = np.arange(E, dtype=np.int64) - indptr[owner]
        d_e, n_e = deg[owner], n[owner]
        # stratified choice of n distinct slots out of deg: slot k from
        # [k*deg//n, (k+1)*deg//n); all slots when deg <= fanout
        lo = (k * d_e) // n_e
        hi = ((k + 1) * d_e) // n_e
        c = (np.uint64(batch) << np.uint64(44)) + (np.uint64(hop) << np.uint64(40)) \
            + np.arange(E, dtype=np.uint64)
        slot = lo + (mix64(key + c) % (hi - lo).astype(np.uint64)).astype(np.int64)
        indices = graph.neighbor(dst[owner], slot)
        blocks.append(Block(dst=dst, indptr=indptr, indices=indices.astype(np.int64)))
        frontier = np.unique(np.concatenate([dst, indices]))
    return blocks, frontier


def full_csr(graph, self_loops: bool = True, chunk: int = 1 << 18):
    """Materialise the whole implicit graph as CSR lists (for graphs small
    enough to hold): node u lists all ``degree(u)`` neighbour slots in slot
    order, preceded by u itself when ``self_loops``.  Returns (indptr,
    indices), int64."""
    N = graph.N
    extra = 1 if self_loops else 0
    deg = graph.degree(np.arange(N, dtype=np.int64)) + extra
    indptr = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    indices = np.empty(int(indptr[-1]), dtype=np.int64)
    for u0 in range(0, N, chunk):
        u1 = min(N, u0 + chunk)
        u = np.arange(u0, u1, dtype=np.int64)
        n = deg[u0:u1]
        owner = np.repeat(u, n)
        k = np.arange(int(indptr[u1] - indptr[u0]), dtype=np.int64) - (indptr[owner] - indptr[u0])
        if self_loops:
            nb = np.where(k == 0, owner, graph.neighbor(owner, np.maximum(k - 1, 0)))
        else:
            nb = graph.neighbor(owner, k)
        indices[indptr[u0]:indptr[u1]] = nb
    return indptr, indices
