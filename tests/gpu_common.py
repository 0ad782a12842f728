"""Helpers of the GPU parity tests: build the HIP path and the oracle on the same seeded inputs."""
import numpy as np

from fg_inputs import features, workload as wl


def make_hotpath(*args, **kwargs):
    from paper_2301_07482_amd.pipeline import make_hotpath as mk      # not at import time: CPU tests import this module too
    return mk(*args, **kwargs)


def rings_bytes(*args, **kwargs):
    from paper_2301_07482_amd.pipeline import rings_bytes as rb
    return rb(*args, **kwargs)


def make_oracle_caches(w, capacity=None, t_stale=None):
    from oracle import freshgnn_oracle as O      # imported where it is used: make_hotpath serves bench.py's timed path too
    dims = wl.layer_dims(w)
    return {l: O.HistoricalCache(w.num_nodes, w.cache_capacity if capacity is None else capacity, dims[l],
                                 w.t_stale if t_stale is None else t_stale, w.compute_dtype)
            for l in range(1, w.num_layers)}


def make_oracle_bidirectional(w, buffer_bytes, capacity=None, t_stale=None):
    """The oracle's shared buffer for workload `w`; its rings take the place of `make_oracle_caches`."""
    from oracle import freshgnn_oracle as O
    dims = wl.layer_dims(w)
    L = w.num_layers
    cap = w.cache_capacity if capacity is None else capacity
    return O.BidirectionalCache(w.num_nodes, [cap] * (L - 1), [dims[l] for l in range(1, L)],
                                w.t_stale if t_stale is None else t_stale, w.compute_dtype, buffer_bytes)


def feature_accessor(w):
    dt = np.float32 if w.feat_dtype == "f32" else np.float16
    return lambda ids: features.feature_rows(w.seed, ids, w.feat_dim, dt)


def to_f32(t):
    """Host float32 copy of a device tensor of any float type."""
    return t.float().cpu().numpy()
