"""The five synthetic workloads and their per-iteration inputs.

Each workload stands in for one of the graphs the paper trains on (its dataset
table, Table 1, and the model settings of Section 7.1): a power-law graph of the
same node and edge counts, features of the same width and type, GraphSAGE
depth, hidden size and batch size of the same order, and a historical cache of
the stated capacity. Gradient norms are synthetic (lognormal), because the path
covered here ends before the loss. Everything is a function of one master seed.
"""
from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

from . import rng
from .graph import ChungLuGraph
from .sampler import sample_minibatch


@dataclass(frozen=True)
class Workload:
    name: str
    num_nodes: int
    num_edges: int
    feat_dim: int
    feat_dtype: str            # "f32" | "f16"
    feat_location: str         # "hbm" | "host"
    hidden: int
    fanouts: Tuple[int, ...]   # input side first: block l uses fanouts[l-1]
    batch: int
    train_nodes: Optional[int]  # size of the training subset seeds are drawn from (None: all nodes)
    cache_capacity: int        # slots per cached layer
    t_stale: int
    p_grad: float
    compute_dtype: str         # "f32" | "bf16": type of H(l>=1), W and the cache rows
    iterations: int
    seed: int = 2301_07482

    @property
    def num_layers(self):
        return len(self.fanouts)

    def scaled(self, factor):
        """Same shape per mini-batch, `factor` times fewer nodes/edges/cache slots (for boxes that cannot hold the table)."""
        return replace(self, name=f"{self.name}/scale{factor}", num_nodes=max(self.batch * 4, self.num_nodes // factor),
                       num_edges=max(1, self.num_edges // factor),
                       train_nodes=None if self.train_nodes is None else max(self.batch, self.train_nodes // factor),
                       cache_capacity=max(1, self.cache_capacity // factor))


WORKLOADS = {
    "tiny": Workload("tiny", 10_000, 100_000, 64, "f32", "hbm", 64, (10, 5), 256, None, 2_000, 10, 0.5, "f32", 20),
    "medium": Workload("medium", 2_400_000, 120_000_000, 100, "f32", "hbm", 256, (15, 10, 5), 1024, None,
                       480_000, 20, 0.3, "f32", 60),
    "large_hbm": Workload("large_hbm", 111_000_000, 1_600_000_000, 128, "f32", "hbm", 256, (15, 10, 5), 1024,
                          1_100_000, 11_100_000, 20, 0.3, "f32", 60),
    "large_host": Workload("large_host", 111_000_000, 1_600_000_000, 128, "f32", "host", 256, (15, 10, 5), 1024,
                           1_100_000, 11_100_000, 20, 0.3, "f32", 60),
    "very_large": Workload("very_large", 244_000_000, 1_700_000_000, 768, "f16", "host", 1024, (25, 15), 1024,
                           1_100_000, 36_600_000, 30, 0.3, "bf16", 80),
}


def layer_dims(w: Workload):
    """d_0 .. d_L: widths of H(0) .. H(L); the last layer keeps the hidden width."""
    return [w.feat_dim] + [w.hidden] * w.num_layers


def make_graph(w: Workload):
    return ChungLuGraph(w.num_nodes, w.num_edges, w.seed)


def seed_nodes(w: Workload, it: int):
    """The `batch` distinct seed nodes of iteration `it` (an epoch is a random permutation of the training subset)."""
    m = w.train_nodes or w.num_nodes
    per_epoch = max(1, m // w.batch)
    epoch, b = divmod(it, per_epoch)
    key = rng.make_key(w.seed, 0x5EED, epoch)
    a = (int(rng.u64(key, 0)) % m) | 1
    import math
    while math.gcd(a, m) != 1:
        a += 2
    off = int(rng.u64(key, 1)) % m
    idx = (np.arange(b * w.batch, (b + 1) * w.batch, dtype=np.uint64) * np.uint64(a % m) + np.uint64(off)) % np.uint64(m)
    # the training subset is the image of [0, m) under a fixed affine bijection of [0, N)
    n = w.num_nodes
    ks = rng.make_key(w.seed, 0x7EA1)
    a2 = (int(rng.u64(ks, 0)) % n) | 1
    while math.gcd(a2, n) != 1:
        a2 += 2
    off2 = int(rng.u64(ks, 1)) % n
    return ((idx * np.uint64(a2 % n) + np.uint64(off2)) % np.uint64(n)).astype(np.int64)


def minibatch(w: Workload, graph, it: int):
    return sample_minibatch(graph, seed_nodes(w, it), w.fanouts, rng.make_key(w.seed, 0x5A3, it))


def grad_norms(w: Workload, it: int, layer: int, node_ids):
    """Synthetic embedding-gradient L2 norms, exp(N(0,1)), keyed by (iteration, layer, node id); fp32."""
    key = rng.make_key(w.seed, 0x6AD, it, layer)
    return np.exp(rng.normal(key, np.asarray(node_ids, dtype=np.int64))).astype(np.float32)


def node_labels(w: Workload, node_ids):
    """Synthetic class of a node, a fixed function of its id, in [0, d_L) (the last layer's width stands for the classes)."""
    key = rng.make_key(w.seed, 0x1ABE1)
    return (rng.u64(key, np.asarray(node_ids, dtype=np.int64)) % np.uint64(layer_dims(w)[-1])).astype(np.int32)


def _round_bf16(x32):
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    b = np.asarray(x32, dtype=np.float32).view(np.uint32)
    r = ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def layer_weights(w: Workload, layer: int):
    """W_l [2*d_{l-1}, d_l] (rows 0..d-1 multiply the node's own row, the rest the neighbour mean) and b_l [d_l].

    Entries are N(0, 1/fan_in) with fan_in = 2*d_{l-1}; bias N(0, 0.01). fp32 values; for the bf16
    workload the weights are pre-rounded to bf16-representable fp32 values (the bias stays fp32).
    """
    dims = layer_dims(w)
    d_in, d_out = dims[layer - 1], dims[layer]
    kw = rng.make_key(w.seed, 0x3E1, layer)
    W = rng.normal(kw, np.arange(2 * d_in * d_out)).reshape(2 * d_in, d_out) / np.sqrt(2.0 * d_in)
    b = 0.1 * rng.normal(rng.make_key(w.seed, 0xB1A5, layer), np.arange(d_out))
    W = W.astype(np.float32)
    if w.compute_dtype == "bf16":
        W = _round_bf16(W)
    return W, b.astype(np.float32)
