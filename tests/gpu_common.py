"""Helpers of the GPU parity tests: build the HIP path and the oracle on the same seeded inputs."""
import numpy as np

from fg_inputs import features, workload as wl
from oracle import freshgnn_oracle as O


def make_hotpath(w, feat_table=None, use_cache=True, capacity=None, t_stale=None, p_grad=None, fused_input=False, one_launch_top_down=True, update_all=True, log_ring=256,
                 hot_ids=None, buffer_bytes=None, backward=False, weight_grads=False, stabilization=0, model="sage"):
    """HotPath for workload `w` with its feature table resident where the workload says."""
    from fg_inputs import device as fdev
    from paper_2301_07482_amd.pipeline import HotPath
    dims = wl.layer_dims(w)
    weights = {l: wl.layer_weights(w, l) for l in range(1, w.num_layers + 1)}
    if model == "gcn":      # one weight matrix per layer: the first d_in rows of the generated pair of panels
        weights = {l: (np.ascontiguousarray(W[:dims[l - 1]]), b) for l, (W, b) in weights.items()}
    if feat_table is None:
        feat_table = fdev.feature_table(w.seed, w.num_nodes, w.feat_dim, w.feat_dtype, w.feat_location)
    hp = HotPath(w.num_nodes, dims, w.fanouts, w.batch, w.cache_capacity if capacity is None else capacity,
                 w.t_stale if t_stale is None else t_stale, w.p_grad if p_grad is None else p_grad, feat_table,
                 w.feat_dtype, w.compute_dtype, weights, features_on_host=(w.feat_location == "host"),
                 use_cache=use_cache, fused_input=fused_input, one_launch_top_down=one_launch_top_down, update_all=update_all,
                 fetch_all=update_all, log_ring=log_ring, hot_ids=hot_ids, buffer_bytes=buffer_bytes, backward=backward, weight_grads=weight_grads, stabilization=stabilization, model=model)
    return hp, weights, feat_table


def make_oracle_caches(w, capacity=None, t_stale=None):
    dims = wl.layer_dims(w)
    return {l: O.HistoricalCache(w.num_nodes, w.cache_capacity if capacity is None else capacity, dims[l],
                                 w.t_stale if t_stale is None else t_stale, w.compute_dtype)
            for l in range(1, w.num_layers)}


def rings_bytes(w, capacity=None):
    """Bytes the rings of workload `w` take at the left end of a shared buffer (each ring starts at a multiple of 256)."""
    dims, es = wl.layer_dims(w), 4 if w.compute_dtype == "f32" else 2
    at = 0
    for l in range(1, w.num_layers):
        at = -(-at // 256) * 256 + (w.cache_capacity if capacity is None else capacity) * dims[l] * es
    return at


def make_oracle_bidirectional(w, buffer_bytes, capacity=None, t_stale=None):
    """The oracle's shared buffer for workload `w`; its rings take the place of `make_oracle_caches`."""
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
