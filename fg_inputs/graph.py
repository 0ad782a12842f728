"""Synthetic graphs for the mini-batch sampler.

Two graph classes offer the same two queries, `degree(v)` and
`neighbour(v, slot)` (the slot-th in-neighbour of v, 0 <= slot < degree(v)):

* `ChungLuGraph`: a directed Chung-Lu power-law graph that is never stored.
  Node ranks r = 0..N-1 carry expected degrees w(r) = c * (r + r0)**(-1/(gamma-1))
  scaled so that sum(w) = num_edges. The in-degree of a node is w rounded up or
  down at random (expectation w), and every in-neighbour slot is an independent
  draw from the distribution proportional to w (inverse CDF of the continuous
  power law), which is the Chung-Lu edge model for a directed graph. Both are
  pure functions of (seed, node[, slot]), so the 1.6-billion-edge graphs of the
  large workloads cost no memory. Node ids are ranks passed through an affine
  bijection so that hubs are not neighbours in memory.
  Parallel edges and self loops can occur among the slots; the sampler drops
  them per row.

* `ExplicitGraph`: an in-neighbour CSR held in memory, for small test graphs.
"""
import math

import numpy as np

from . import rng


class ExplicitGraph:
    def __init__(self, indptr, indices):
        self.indptr = np.asarray(indptr, dtype=np.int64)
        self.indices = np.asarray(indices, dtype=np.int64)
        self.num_nodes = self.indptr.shape[0] - 1

    def degree(self, v):
        v = np.asarray(v, dtype=np.int64)
        return self.indptr[v + 1] - self.indptr[v]

    def access_estimate(self):
        """How often each node is named as an in-neighbour: what a uniform neighbour sampler visits in proportion to."""
        return np.bincount(self.indices, minlength=self.num_nodes).astype(np.float64)

    def neighbour(self, v, slot):
        v = np.asarray(v, dtype=np.int64)
        if self.indices.shape[0] == 0:
            return np.zeros(np.broadcast(v, slot).shape, dtype=np.int64)
        # slots past a row's degree are the caller's to mask; keep the index in range
        at = np.minimum(self.indptr[v] + np.asarray(slot, dtype=np.int64), self.indices.shape[0] - 1)
        return self.indices[at]


class ChungLuGraph:
    def __init__(self, num_nodes, num_edges, seed, gamma=2.5):
        self.num_nodes = int(num_nodes)
        self.num_edges = int(num_edges)
        self.seed = int(seed)
        self.alpha = 1.0 / (gamma - 1.0)
        self.r0 = max(1.0, 1e-6 * self.num_nodes)
        e = 1.0 - self.alpha
        self._e = e
        self._lo = self.r0 ** e
        self._span = (self.num_nodes + self.r0) ** e - self._lo
        self.c = self.num_edges * e / self._span
        self._key_deg = rng.make_key(seed, 0xDE6)
        self._key_nbr = rng.make_key(seed, 0x4B12)
        # affine bijection rank -> id on [0, N)
        n = self.num_nodes
        a = int(0.6180339887 * n) | 1
        while math.gcd(a, n) != 1:
            a += 2
        self._a = a % n if n > 1 else 0
        self._ainv = pow(self._a, -1, n) if n > 1 else 0
        self._b = int(rng.u64(rng.make_key(seed, 0xB1), 0)) % n

    def rank_to_id(self, r):
        r = np.asarray(r).astype(np.uint64)
        return ((r * np.uint64(self._a) + np.uint64(self._b)) % np.uint64(self.num_nodes)).astype(np.int64)

    def id_to_rank(self, v):
        n = np.uint64(self.num_nodes)
        v = np.asarray(v).astype(np.uint64)
        return (((v + n - np.uint64(self._b)) % n) * np.uint64(self._ainv) % n).astype(np.int64)

    def expected_degree(self, v):
        r = self.id_to_rank(v).astype(np.float64)
        return self.c * (r + 0.5 + self.r0) ** (-self.alpha)

    def access_estimate(self, v):
        """Proportional to the probability that a neighbour slot names v (every slot is a draw proportional to w)."""
        return self.expected_degree(v)

    def hottest(self, count):
        """The `count` nodes with the largest access estimate, largest first: w falls strictly with the rank."""
        return self.rank_to_id(np.arange(min(int(count), self.num_nodes), dtype=np.int64)).astype(np.int32)

    def degree(self, v):
        v = np.asarray(v, dtype=np.int64)
        w = self.expected_degree(v)
        fl = np.floor(w)
        u = rng.uniform(rng.u64(self._key_deg, v))
        return (fl + (u < (w - fl))).astype(np.int64)

    def neighbour(self, v, slot):
        v = np.asarray(v, dtype=np.int64)
        u = rng.uniform(rng.u64_2(self._key_nbr, v, np.asarray(slot, dtype=np.int64)))
        x = (self._lo + u * self._span) ** (1.0 / self._e) - self.r0
        r = np.clip(np.floor(x), 0, self.num_nodes - 1).astype(np.int64)
        return self.rank_to_id(r)
