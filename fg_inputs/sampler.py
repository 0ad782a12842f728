"""Uniform neighbour sampler producing the layered mini-batch both sides consume.

Layout of a sampled L-layer mini-batch (layer L = seeds, layer 0 = input nodes):

* `ids[l]`, l = 0..L: distinct node ids of layer l (int32). Layer l-1 starts
  with the nodes of layer l in the same order (a node needs its own previous
  embedding), followed by newly sampled neighbours in order of first occurrence.
* block l, l = 1..L, connects layer l-1 (sources) to layer l (rows) with two
  row arrays: the neighbours of row j are `col[l][start[l][j] : end[l][j]]`,
  each a position into `ids[l-1]`. Setting `end[j] = start[j]` removes the
  neighbours of row j without touching `col`.

Per row, min(degree, fanout) neighbour slots are chosen (all of them when the
degree does not exceed the fan-out, otherwise one slot from each of `fanout`
disjoint strata of the slot range with integer bounds, the whole choice then
turned round the row by a common random offset, which gives `fanout` distinct
slots and every slot the same inclusion probability); self loops and repeated
neighbours within the row are dropped.
`fanouts` lists the fan-out from the input side to the seed side: block l uses
`fanouts[l - 1]`.

This is input generation only; it contains none of the cache or model logic.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import rng


@dataclass
class MiniBatch:
    num_layers: int
    ids: List[np.ndarray]                      # index 0..L
    start: List[Optional[np.ndarray]]          # index 1..L (0 unused)
    end: List[Optional[np.ndarray]]
    col: List[Optional[np.ndarray]]
    meta: dict = field(default_factory=dict)

    def copy(self):
        cp = lambda xs: [None if x is None else x.copy() for x in xs]
        return MiniBatch(self.num_layers, cp(self.ids), cp(self.start), cp(self.end), cp(self.col), dict(self.meta))


def sample_minibatch(graph, seeds, fanouts, key):
    L = len(fanouts)
    ids = [None] * (L + 1)
    start = [None] * (L + 1)
    end = [None] * (L + 1)
    col = [None] * (L + 1)
    cur = np.asarray(seeds, dtype=np.int64)
    assert np.unique(cur).shape[0] == cur.shape[0], "seed nodes must be distinct"
    ids[L] = cur
    for l in range(L, 0, -1):
        f = int(fanouts[l - 1])
        n = cur.shape[0]
        deg = graph.degree(cur)
        j = np.arange(f, dtype=np.int64)[None, :]
        key_l = rng.make_key(key, l)
        u = rng.uniform(rng.u64_2(key_l, cur[:, None], j))
        dcol = deg[:, None].astype(np.int64)
        first = (j * dcol) // f
        width = np.maximum(((j + 1) * dcol) // f - first, 1)
        inside = np.minimum(np.floor(u * width).astype(np.int64), width - 1)
        turn = np.floor(rng.uniform(rng.u64_2(key_l, cur, np.int64(f))) * deg).astype(np.int64)
        turn = np.minimum(turn, np.maximum(deg - 1, 0))[:, None]
        strat = (first + inside + turn) % np.maximum(dcol, 1)
        slot = np.where(dcol <= f, j, strat)
        valid = j < np.minimum(deg, f)[:, None]
        slot = np.where(valid, np.minimum(slot, np.maximum(dcol - 1, 0)), 0)
        nb = np.where(valid, graph.neighbour(np.broadcast_to(cur[:, None], slot.shape), slot), -1)
        valid &= nb != cur[:, None]
        for a in range(1, f):
            for b in range(a):
                valid[:, a] &= ~(valid[:, b] & (nb[:, a] == nb[:, b]))
        cnt = valid.sum(axis=1)
        st = np.zeros(n, dtype=np.int64)
        if n:
            st[1:] = np.cumsum(cnt)[:-1]
        cand = nb[valid]
        allv = np.concatenate([cur, cand])
        uniq, first, inv = np.unique(allv, return_index=True, return_inverse=True)
        order = np.argsort(first, kind="stable")
        pos_of_uniq = np.empty(uniq.shape[0], dtype=np.int64)
        pos_of_uniq[order] = np.arange(uniq.shape[0], dtype=np.int64)
        pos = pos_of_uniq[inv]
        prev = uniq[order]
        assert prev.shape[0] < 2 ** 31 and cand.shape[0] < 2 ** 31
        start[l] = st.astype(np.int32)
        end[l] = (st + cnt).astype(np.int32)
        col[l] = pos[n:].astype(np.int32)
        ids[l - 1] = prev
        cur = prev
    ids = [x.astype(np.int32) for x in ids]
    return MiniBatch(L, ids, start, end, col)



def transpose_block(start, end, col, n_src):
    """The transpose of one sampled block: for every source position j the rows that sampled it, as
    (t_start[j], t_end[j]) into t_row, rows in ascending order. Built from the block as sampled (before any pruning)."""
    start = np.asarray(start, dtype=np.int64)
    end = np.asarray(end, dtype=np.int64)
    deg = end - start
    rows = np.repeat(np.arange(len(start), dtype=np.int64), deg)
    within = np.arange(len(rows), dtype=np.int64) - np.repeat(np.cumsum(deg) - deg, deg)
    src = np.asarray(col, dtype=np.int64)[np.repeat(start, deg) + within] if len(rows) else np.zeros(0, dtype=np.int64)
    order = np.argsort(src, kind="stable")
    counts = np.bincount(src, minlength=n_src)
    t_end = np.cumsum(counts)
    t_start = t_end - counts
    return t_start.astype(np.int32), t_end.astype(np.int32), rows[order].astype(np.int32)
