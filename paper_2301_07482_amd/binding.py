"""Thin ctypes binding of libfreshgnn.so: same names as the C ABI, argument marshalling only.

Tensors are passed as raw device pointers (torch is used for device memory and streams, nothing
else); every step runs in the library's HIP kernels. There is no fallback: if the shared library is
missing, importing this module raises.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfreshgnn.so")

FG_OK, FG_ERR_INVALID_ARG, FG_ERR_SHAPE, FG_ERR_DTYPE, FG_ERR_STATE, FG_ERR_OOM, FG_ERR_HIP = range(7)
FG_F32, FG_F16, FG_BF16 = 0, 1, 2
FG_WS_LOOKUP_PRUNE, FG_WS_CACHE_UPDATE, FG_WS_EXPORT = 0, 1, 2
FG_TABLE_HBM_STREAMED, FG_TABLE_HOST_MAPPED, FG_TABLE_HBM_REUSED = 0, 1, 2
DTYPE_SIZE = {FG_F32: 4, FG_F16: 2, FG_BF16: 2}

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2301_07482_amd.build` (needs hipcc); "
                      "there is no fallback implementation")
_lib = C.CDLL(LIB_PATH)

_p, _i32, _i64, _sz, _f = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float

SIGNATURES = {
    "fg_last_error": (C.c_char_p, []),
    "fg_version": (_i32, []),
    "fg_cache_create": (_i32, [C.POINTER(_p), _i64, _i32, C.POINTER(_i64), C.POINTER(_i32), _i32, _i32, _p]),
    "fg_cache_create_bidirectional": (_i32, [C.POINTER(_p), _i64, _i32, C.POINTER(_i64), C.POINTER(_i32), _i32, _i32, _i64, _p]),
    "fg_cache_fill_features": (_i32, [_p, _p, _i64, _p, _i64, _i64, _i64, _p]),
    "fg_feature_lookup": (_i32, [_p, _p, _p, _i64, _p, _p, _p]),
    "fg_cache_buffer": (_p, [_p, C.POINTER(_i64)]),
    "fg_cache_feature_rows": (_i64, [_p]),
    "fg_cache_ring_offset": (_i64, [_p, _i32]),
    "fg_gather_features": (_i32, [_p, _p, _i64, _i64, _i64, _p, _p, _p, _i64, _p, _i64, _i64, _i32, _p]),
    "fg_gather_aggregate_features": (_i32, [_p, _p, _p, _p, _i64, _i32, _p, _p, _i64, _p, _i32, _p, _i64, _i64, _i32, _i32, _p,
                                            _i64, _i32, _p, _i64, _i32, _p]),
    "fg_cache_destroy": (_i32, [_p]),
    "fg_cache_clear": (_i32, [_p, _p]),
    "fg_cache_table": (_p, [_p, _i32]),
    "fg_cache_set_t_stale": (_i32, [_p, _i32]),
    "fg_cache_set_stabilization": (_i32, [_p, _i64]),
    "fg_cache_export": (_i32, [_p, _i32, _i64, _p, _p, _p, _p, _p, _p, _sz, _p]),
    "fg_workspace_bytes": (_sz, [_i32, _i64, _i64]),
    "fg_set_tuning": (_i32, [C.c_char_p, _i64]),
    "fg_lookup_prune": (_i32, [_p, _i32, _i64, _p, _i32, _p, _p, _p, _p, _i64, _i32, _p, _p, _p, _p, _p, _p, _p, _p, _sz, _p]),
    "fg_lookup_prune_static": (_i32, [_p, _i32, _i64, _p, _i32, _p, _p, _p, _p, _i64, _i32, _p, _p, _p, _p, _p, _p, _p, _p]),
    "fg_gather": (_i32, [_p, _i64, _i64, _i64, _p, _p, _p, _i64, _p, _i64, _i64, _i32, _p]),
    "fg_aggregate": (_i32, [_p, _p, _p, _i64, _i32, _p, _p, _i64, _p, _i32, _i64, _i32, _i32, _p, _i64, _i32, _p]),
    "fg_gather_aggregate": (_i32, [_p, _p, _p, _i64, _i32, _p, _p, _i64, _p, _i32, _p, _i64, _i64, _i32, _i32, _p, _i64, _i32,
                                   _p, _i64, _i32, _p]),
    "fg_aggregate_gcn": (_i32, [_p, _p, _p, _i64, _i32, _p, _p, _i64, _p, _i32, _i64, _i32, _p, _p, _p]),
    "fg_gather_aggregate_gcn": (_i32, [_p, _p, _p, _i64, _i32, _p, _p, _i64, _p, _i32, _p, _i64, _i64, _i32, _p, _p, _p]),
    "fg_sample_block_workspace_bytes": (_sz, [_i64, _i32]),
    "fg_sample_block": (_i32, [_p, _p, _i64, _i64, _p, _p, _i64, _i32, C.c_uint64, _i32, _p, _p, _p, _p, _p, _i64, _p, _p, _sz, _p]),
    "fg_transpose_block_workspace_bytes": (_sz, [_i64]),
    "fg_transpose_block": (_i32, [_p, _p, _p, _p, _i64, _p, _i64, _i64, _p, _p, _p, _p, _sz, _p]),
    "fg_access_estimate": (_i32, [_p, _p, _p, _i64, _i32, _p, _p, _i32, _p, _p]),
    "fg_gather_aggregate_ids": (_i32, [_p, _p, _p, _i64, _i32, _p, _p, _i64, _p, _p, _i64, _i64, _i32, _i32, _p, _i64, _i32, _p, _i64,
                                       _i32, _p, _i32, _p, _p]),
    "fg_linear": (_i32, [_p, _i32, _i64, _i32, _p, _i64, _p, _p, _i64, _i32, _i32, _p, _i32, _p, _i32, _p, _i32, _i64, _i32, _p]),
    "fg_linear_wt": (_i32, [_p, _i32, _i64, _i32, _p, _i64, _p, _p, _i64, _i32, _i32, _p, _i32, _p, _i32, _p, _i32, _i64, _i32, _p]),
    "fg_linear_ids": (_i32, [_p, _i32, _i64, _i32, _p, _p, _i64, _p, _p, _i64, _i32, _i32, _p, _i32, _p, _i32, _p, _i32, _i64, _i32, _p]),
    "fg_aggregate_linear": (_i32, [_p, _p, _p, _i64, _i32, _p, _p, _i64, _p, _i32, _i64, _i32, _i32, _p, _p, _i32, _p, _i64, _p, _i32,
                                   _i64, _p]),
    "fg_cache_update": (_i32, [_p, _i32, _i64, _p, _i32, _p, _p, _p, _f, _p, _i64, _p, _p, _sz, _p]),
    "fg_softmax_xent_grad": (_i32, [_p, _i64, _p, _i32, _i32, _p, _i64, _p]),
    "fg_row_norms": (_i32, [_p, _i64, _i32, _i32, _p, _p]),
    "fg_layer_backward_workspace_bytes": (_sz, [_i32, _i64, _i32, _i32]),
    "fg_layer_backward_weights_workspace_bytes": (_sz, [_i64, _i32, _i32]),
    "fg_layer_backward_weights": (_i32, [_p, _i32, _i64, _p, _i64, _p, _i64, _p, _i64, _i32, _p, _p, _i64, _i32, _i32, _p, _p, _p, _sz, _p]),
    "fg_layer_backward": (_i32, [_p, _i64, _p, _i64, _i32, _p, _p, _i64, _p, _p, _p, _p, _p, _p, _p, _i64, _i32, _i32, _i32, _p, _p,
                                 _i64, _p, _p, _sz, _p]),
    "fg_layer_backward_gcn_workspace_bytes": (_sz, [_i32, _i64, _i32, _i32]),
    "fg_layer_backward_gcn": (_i32, [_p, _i64, _p, _i64, _i32, _p, _p, _i64, _p, _p, _p, _p, _p, _p, _p, _i64, _i32, _i32, _i32, _p, _p,
                                     _i64, _p, _p, _sz, _p]),
    "fg_layer_backward_bf16_workspace_bytes": (_sz, [_i32, _i64, _i32, _i32]),
    "fg_layer_backward_bf16": (_i32, [_p, _i64, _p, _i64, _i32, _p, _p, _i64, _p, _p, _p, _p, _p, _p, _p, _i64, _i32, _i32, _i32, _p, _p,
                                      _i64, _p, _p, _sz, _p]),
    "fg_layer_backward_weights_bf16_workspace_bytes": (_sz, [_i64, _i32, _i32]),
    "fg_layer_backward_weights_bf16": (_i32, [_p, _i32, _i64, _i32, _p, _i64, _p, _i64, _p, _i64, _i32, _p, _p, _i64, _i32, _i32, _p, _p,
                                              _p, _sz, _p]),
}


class TopDownLayer(C.Structure):
    """fg_top_down_layer_t"""
    _fields_ = [("cache_layer", _i32), ("n", _i32), ("ids_dev", _p), ("live_dev", _p), ("row_start_dev", _p),
                ("row_end_dev", _p), ("col_dev", _p), ("nnz", _i64), ("n_src", _i32), ("live_src_dev", _p), ("hit_dev", _p),
                ("hit_pos_dev", _p), ("hit_slot_dev", _p), ("normal_pos_dev", _p), ("normal_ids_dev", _p), ("counts_dev", _p), ("n_dev", _p)]


SIGNATURES["fg_top_down_workspace_bytes"] = (_sz, [_i32, C.POINTER(TopDownLayer)])
SIGNATURES["fg_top_down"] = (_i32, [_p, _i64, _i32, C.POINTER(TopDownLayer), _p, _sz, _p])



class UpdateLayer(C.Structure):
    """fg_update_layer_t"""
    _fields_ = [("layer", _i32), ("n", _i32), ("ids_dev", _p), ("live_dev", _p), ("hit_dev", _p), ("gnorm_dev", _p),
                ("h_dev", _p), ("h_stride", _i64), ("stats_dev", _p), ("saving_dev", _p), ("max_admit", _i64), ("n_dev", _p)]


class FetchLayer(C.Structure):
    """fg_fetch_layer_t"""
    _fields_ = [("layer", _i32), ("hit_slot_dev", _p), ("hit_pos_dev", _p), ("n_hit_dev", _p), ("max_hits", _i64),
                ("h_dev", _p), ("h_rows", _i64), ("h_stride", _i64)]


SIGNATURES["fg_cache_fetch_all"] = (_i32, [_p, _i32, C.POINTER(FetchLayer), _p])
SIGNATURES["fg_cache_update_all"] = (_i32, [_p, _i64, _f, _i32, C.POINTER(UpdateLayer), _p, _sz, _p])
SIGNATURES["fg_cache_update_select"] = (_i32, [_p, _i64, _f, _i32, C.POINTER(UpdateLayer), _p, _sz, _p])
SIGNATURES["fg_cache_update_commit"] = (_i32, [_p, _i64, _i32, C.POINTER(UpdateLayer), _p, _sz, _p])

for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(_lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


class FgError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"freshgnn error {code}: {message}")
        self.code = code


def _check(rc):
    if rc != FG_OK:
        raise FgError(rc, _lib.fg_last_error().decode())


def ptr(t):
    """Raw address of a torch tensor (or None); an int is passed through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def fg_version():
    return _lib.fg_version()


def fg_last_error():
    return _lib.fg_last_error().decode()


def fg_set_tuning(key, value):
    _check(_lib.fg_set_tuning(key.encode(), value))


def fg_workspace_bytes(kind, n):
    return _lib.fg_workspace_bytes(kind, n, 0)


def fg_cache_create(num_nodes, capacity, dim, dtype, t_stale, stream=None):
    n = len(capacity)
    handle = _p()
    cap = (_i64 * max(n, 1))(*capacity)
    dm = (_i32 * max(n, 1))(*dim)
    _check(_lib.fg_cache_create(C.byref(handle), num_nodes, n, cap, dm, dtype, t_stale, stream))
    return handle


def fg_cache_create_bidirectional(num_nodes, capacity, dim, dtype, t_stale, buffer_bytes, stream=None):
    n = len(capacity)
    handle = _p()
    cap = (_i64 * max(n, 1))(*capacity)
    dm = (_i32 * max(n, 1))(*dim)
    _check(_lib.fg_cache_create_bidirectional(C.byref(handle), num_nodes, n, cap, dm, dtype, t_stale, buffer_bytes, stream))
    return handle


def fg_cache_fill_features(cache, hot_ids, n_hot, table, table_rows, src_stride, row_bytes, stream=None):
    _check(_lib.fg_cache_fill_features(cache, ptr(hot_ids), n_hot, ptr(table), table_rows, src_stride, row_bytes, stream))


def fg_feature_lookup(cache, ids, count, max_count, rank_out, n_found, stream=None):
    _check(_lib.fg_feature_lookup(cache, ptr(ids), ptr(count), max_count, ptr(rank_out), ptr(n_found), stream))


def fg_cache_buffer(cache):
    """(device address, bytes) of the buffer embeddings and raw features share."""
    n = _i64(0)
    return _lib.fg_cache_buffer(cache, C.byref(n)), n.value


def fg_cache_feature_rows(cache):
    return _lib.fg_cache_feature_rows(cache)


def fg_cache_ring_offset(cache, layer):
    return _lib.fg_cache_ring_offset(cache, layer)


def fg_cache_destroy(cache):
    _check(_lib.fg_cache_destroy(cache))


def fg_cache_clear(cache, stream=None):
    _check(_lib.fg_cache_clear(cache, stream))


def fg_cache_table(cache, layer):
    return _lib.fg_cache_table(cache, layer)


def fg_cache_set_t_stale(cache, t_stale):
    _check(_lib.fg_cache_set_t_stale(cache, t_stale))


def fg_cache_set_stabilization(cache, n_iterations):
    _check(_lib.fg_cache_set_stabilization(cache, n_iterations))


def fg_cache_export(cache, layer, it, nodes, slots, stamps, count, head, ws, ws_bytes, stream=None):
    _check(_lib.fg_cache_export(cache, layer, it, ptr(nodes), ptr(slots), ptr(stamps), ptr(count), ptr(head), ptr(ws),
                                ws_bytes, stream))


def fg_lookup_prune(cache, layer, it, ids, n, live, row_start, row_end, col, nnz, n_src, live_src, hit, hit_pos, hit_slot,
                    normal_pos, normal_ids, counts, ws, ws_bytes, stream=None):
    _check(_lib.fg_lookup_prune(cache, layer, it, ptr(ids), n, ptr(live), ptr(row_start), ptr(row_end), ptr(col), nnz, n_src,
                                ptr(live_src), ptr(hit), ptr(hit_pos), ptr(hit_slot), ptr(normal_pos), ptr(normal_ids),
                                ptr(counts), ptr(ws), ws_bytes, stream))


FG_LOOKUP_PRUNE_STATIC_MAX_N = 2097152


def fg_lookup_prune_static(cache, layer, it, ids, n, live, row_start, row_end, col, nnz, n_src, live_src, hit, hit_pos, hit_slot,
                           normal_pos, normal_ids, counts, stream=None):
    _check(_lib.fg_lookup_prune_static(cache, layer, it, ptr(ids), n, ptr(live), ptr(row_start), ptr(row_end), ptr(col), nnz,
                                       n_src, ptr(live_src), ptr(hit), ptr(hit_pos), ptr(hit_slot), ptr(normal_pos),
                                       ptr(normal_ids), ptr(counts), stream))


def top_down_layers(specs):
    """ctypes array of fg_top_down_layer_t from dicts (tensors or addresses; missing keys are NULL / 0)."""
    return _struct_array(TopDownLayer, specs)


def fg_top_down_workspace_bytes(layers):
    return _lib.fg_top_down_workspace_bytes(len(layers), layers)


def fg_top_down(cache, it, layers, ws, ws_bytes, stream=None):
    _check(_lib.fg_top_down(cache, it, len(layers), layers, ptr(ws), ws_bytes, stream))


def fg_gather(table, table_rows, src_stride, row_bytes, src_index, dst_pos, count, max_count, dst, dst_rows, dst_stride,
              table_kind=0, stream=None):
    _check(_lib.fg_gather(ptr(table), table_rows, src_stride, row_bytes, ptr(src_index), ptr(dst_pos), ptr(count), max_count,
                          ptr(dst), dst_rows, dst_stride, table_kind, stream))


def fg_gather_features(cache, table, table_rows, src_stride, row_bytes, ids, dst_pos, count, max_count, dst, dst_rows, dst_stride,
                       table_kind=0, stream=None):
    _check(_lib.fg_gather_features(cache, ptr(table), table_rows, src_stride, row_bytes, ptr(ids), ptr(dst_pos), ptr(count),
                                   max_count, ptr(dst), dst_rows, dst_stride, table_kind, stream))


def fg_aggregate(row_start, row_end, col, nnz, n_block_rows, rows, n_rows, max_rows, h_src, n_src, src_stride, dim, in_dtype,
                 agg, agg_stride, out_dtype, stream=None):
    _check(_lib.fg_aggregate(ptr(row_start), ptr(row_end), ptr(col), nnz, n_block_rows, ptr(rows), ptr(n_rows), max_rows,
                             ptr(h_src), n_src, src_stride, dim, in_dtype, ptr(agg), agg_stride, out_dtype, stream))


def fg_gather_aggregate(row_start, row_end, col, nnz, n_block_rows, rows, n_rows, max_rows, src_ids, n_src, table, table_rows,
                        src_stride, dim, in_dtype, agg, agg_stride, out_dtype, h_self_out=None, h_self_stride=0, n_self_rows=0,
                        stream=None):
    _check(_lib.fg_gather_aggregate(ptr(row_start), ptr(row_end), ptr(col), nnz, n_block_rows, ptr(rows), ptr(n_rows), max_rows,
                                    ptr(src_ids), n_src, ptr(table), table_rows, src_stride, dim, in_dtype, ptr(agg),
                                    agg_stride, out_dtype, ptr(h_self_out), h_self_stride, n_self_rows, stream))


def fg_gather_aggregate_features(cache, row_start, row_end, col, nnz, n_block_rows, rows, n_rows, max_rows, src_ids, n_src, table,
                                 table_rows, src_stride, dim, in_dtype, agg, agg_stride, out_dtype, h_self_out=None,
                                 h_self_stride=0, n_self_rows=0, stream=None):
    _check(_lib.fg_gather_aggregate_features(cache, ptr(row_start), ptr(row_end), ptr(col), nnz, n_block_rows, ptr(rows),
                                             ptr(n_rows), max_rows, ptr(src_ids), n_src, ptr(table), table_rows, src_stride, dim,
                                             in_dtype, ptr(agg), agg_stride, out_dtype, ptr(h_self_out), h_self_stride,
                                             n_self_rows, stream))


def fg_aggregate_gcn(row_start, row_end, col, nnz, n_block_rows, rows, n_rows, max_rows, h_src, n_src, src_stride, dim, mean_pos,
                     mean_cmp, stream=None):
    _check(_lib.fg_aggregate_gcn(ptr(row_start), ptr(row_end), ptr(col), nnz, n_block_rows, ptr(rows), ptr(n_rows), max_rows,
                                 ptr(h_src), n_src, src_stride, dim, ptr(mean_pos), ptr(mean_cmp), stream))


def fg_gather_aggregate_gcn(row_start, row_end, col, nnz, n_block_rows, rows, n_rows, max_rows, src_ids, n_src, table, table_rows,
                            src_stride, dim, mean_pos, mean_cmp, stream=None):
    _check(_lib.fg_gather_aggregate_gcn(ptr(row_start), ptr(row_end), ptr(col), nnz, n_block_rows, ptr(rows), ptr(n_rows), max_rows,
                                        ptr(src_ids), n_src, ptr(table), table_rows, src_stride, dim, ptr(mean_pos), ptr(mean_cmp),
                                        stream))


def fg_gather_aggregate_ids(row_start, row_end, col_ids, nnz, n_block_rows, rows, n_rows, max_rows, row_ids, table, table_rows,
                            src_stride, dim, in_dtype, agg, agg_stride, out_dtype, h_self_out=None, h_self_stride=0, n_self_rows=0,
                            cache=None, fetch_layers=None, stream=None):
    """fetch_layers: a `fetch_layers(...)` array (with `cache`) whose copies share the loader's launch, or None."""
    n_fetch = len(fetch_layers) if fetch_layers is not None else 0
    _check(_lib.fg_gather_aggregate_ids(ptr(row_start), ptr(row_end), ptr(col_ids), nnz, n_block_rows, ptr(rows), ptr(n_rows),
                                        max_rows, ptr(row_ids), ptr(table), table_rows, src_stride, dim, in_dtype, ptr(agg),
                                        agg_stride, out_dtype, ptr(h_self_out), h_self_stride, n_self_rows, cache, n_fetch,
                                        C.cast(fetch_layers, _p) if n_fetch else None, stream))


def fg_linear(h_src, n_src, src_stride, in_dtype, agg, agg_stride, rows, n_rows, max_rows, d_in, d_out, W, w_dtype, bias, relu,
              h_out, n_out, out_stride, out_dtype, stream=None):
    _check(_lib.fg_linear(ptr(h_src), n_src, src_stride, in_dtype, ptr(agg), agg_stride, ptr(rows), ptr(n_rows), max_rows,
                          d_in, d_out, ptr(W), w_dtype, ptr(bias), relu, ptr(h_out), n_out, out_stride, out_dtype, stream))


def fg_linear_wt(h_src, n_src, src_stride, in_dtype, agg, agg_stride, rows, n_rows, max_rows, d_in, d_out, Wt, w_dtype, bias, relu,
                 h_out, n_out, out_stride, out_dtype, stream=None):
    _check(_lib.fg_linear_wt(ptr(h_src), n_src, src_stride, in_dtype, ptr(agg), agg_stride, ptr(rows), ptr(n_rows), max_rows,
                             d_in, d_out, ptr(Wt), w_dtype, ptr(bias), relu, ptr(h_out), n_out, out_stride, out_dtype, stream))


def fg_linear_ids(table, table_rows, src_stride, in_dtype, src_ids, agg, agg_stride, rows, n_rows, max_rows, d_in, d_out, W, w_dtype, bias,
                  relu, h_out, n_out, out_stride, out_dtype, stream=None):
    _check(_lib.fg_linear_ids(ptr(table), table_rows, src_stride, in_dtype, ptr(src_ids), ptr(agg), agg_stride, ptr(rows), ptr(n_rows),
                              max_rows, d_in, d_out, ptr(W), w_dtype, ptr(bias), relu, ptr(h_out), n_out, out_stride, out_dtype, stream))


def fg_aggregate_linear(row_start, row_end, col, nnz, n_block_rows, rows, n_rows, max_rows, h_src, n_src, src_stride, d_in, d_out, W,
                        bias, relu, agg_ws, agg_stride, h_out, n_out, out_stride, stream=None):
    _check(_lib.fg_aggregate_linear(ptr(row_start), ptr(row_end), ptr(col), nnz, n_block_rows, ptr(rows), ptr(n_rows), max_rows,
                                    ptr(h_src), n_src, src_stride, d_in, d_out, ptr(W), ptr(bias), relu, ptr(agg_ws), agg_stride,
                                    ptr(h_out), n_out, out_stride, stream))


def one_launch_layer(max_rows, d_in, d_out):
    """Whether fg_aggregate_linear runs a layer of this shape as one launch (the rule stated in freshgnn.h)."""
    return d_in % 32 == 0 and d_in <= 256 and -(-max_rows // 32) * -(-d_out // 32) <= 768


def fg_cache_update(cache, layer, it, ids, n, live, hit, gnorm, p_grad, h, h_stride, stats, ws, ws_bytes, stream=None):
    _check(_lib.fg_cache_update(cache, layer, it, ptr(ids), n, ptr(live), ptr(hit), ptr(gnorm), p_grad, ptr(h), h_stride,
                                ptr(stats), ptr(ws), ws_bytes, stream))


def fg_softmax_xent_grad(h, h_stride, labels, n, d, dh, dh_stride, stream=None):
    _check(_lib.fg_softmax_xent_grad(ptr(h), h_stride, ptr(labels), n, d, ptr(dh), dh_stride, stream))


def fg_row_norms(x, x_stride, n, d, norms, stream=None):
    _check(_lib.fg_row_norms(ptr(x), x_stride, n, d, ptr(norms), stream))


LAYER_BACKWARD_KINDS = {"sage": "fg_layer_backward", "gcn": "fg_layer_backward_gcn", "bf16": "fg_layer_backward_bf16"}


def fg_layer_backward_workspace_bytes(n, max_rows, d_in, d_out, kind="sage"):
    return getattr(_lib, LAYER_BACKWARD_KINDS[kind] + "_workspace_bytes")(n, max_rows, d_in, d_out)


def fg_layer_backward(dh, dh_stride, h, h_stride, n, rows, n_rows, max_rows, live, hit, row_start, row_end, t_start, t_end, t_row,
                      nnz, n_src, d_in, d_out, W, dh_src, dh_src_stride, norms_src, ws, ws_bytes, stream=None, kind="sage"):
    """kind: "sage" = fg_layer_backward, "gcn" = fg_layer_backward_gcn, "bf16" = fg_layer_backward_bf16 (same argument lists)."""
    fn = getattr(_lib, LAYER_BACKWARD_KINDS[kind])
    _check(fn(ptr(dh), dh_stride, ptr(h), h_stride, n, ptr(rows), ptr(n_rows), max_rows, ptr(live), ptr(hit),
              ptr(row_start), ptr(row_end), ptr(t_start), ptr(t_end), ptr(t_row), nnz, n_src, d_in, d_out,
              ptr(W), ptr(dh_src), dh_src_stride, ptr(norms_src), ptr(ws), ws_bytes, stream))


def fg_layer_backward_gcn(*args, **kw):
    fg_layer_backward(*args, kind="gcn", **kw)


def fg_layer_backward_bf16(*args, **kw):
    fg_layer_backward(*args, kind="bf16", **kw)


def fg_layer_backward_weights_workspace_bytes(max_rows, d_in, d_out):
    return _lib.fg_layer_backward_weights_workspace_bytes(max_rows, d_in, d_out)


def fg_layer_backward_weights(h_src, n_src, src_stride, agg, agg_stride, dh, dh_stride, h, h_stride, n, rows, n_rows, max_rows, d_in,
                              d_out, dw, db, ws, ws_bytes, stream=None):
    _check(_lib.fg_layer_backward_weights(ptr(h_src), n_src, src_stride, ptr(agg), agg_stride, ptr(dh), dh_stride, ptr(h), h_stride, n,
                                          ptr(rows), ptr(n_rows), max_rows, d_in, d_out, ptr(dw), ptr(db), ptr(ws), ws_bytes, stream))


def fg_layer_backward_weights_bf16_workspace_bytes(max_rows, d_in, d_out):
    return _lib.fg_layer_backward_weights_bf16_workspace_bytes(max_rows, d_in, d_out)


def fg_layer_backward_weights_bf16(h_src, n_src, src_stride, src_dtype, agg, agg_stride, dh, dh_stride, h, h_stride, n, rows, n_rows,
                                   max_rows, d_in, d_out, dw, db, ws, ws_bytes, stream=None):
    _check(_lib.fg_layer_backward_weights_bf16(ptr(h_src), n_src, src_stride, src_dtype, ptr(agg), agg_stride, ptr(dh), dh_stride, ptr(h),
                                               h_stride, n, ptr(rows), ptr(n_rows), max_rows, d_in, d_out, ptr(dw), ptr(db), ptr(ws),
                                               ws_bytes, stream))


_POINTER_FIELDS = {}


def _struct_array(struct, specs):
    """ctypes array of `struct` from dicts keyed by its field names. A new array is all zero bytes, so a key that is
    missing or None stays NULL / 0; only what a dict holds is written."""
    is_ptr = _POINTER_FIELDS.get(struct)
    if is_ptr is None:
        is_ptr = _POINTER_FIELDS[struct] = {name: ctype is _p for name, ctype in struct._fields_}
    arr = (struct * len(specs))()
    for a, spec in zip(arr, specs):
        for name, v in spec.items():
            if v is None:
                continue
            if is_ptr[name] and not isinstance(v, int):
                v = v.data_ptr()
            setattr(a, name, v)
    return arr


def update_layers(specs):
    """ctypes array of fg_update_layer_t from dicts keyed by the field names (tensors or addresses for pointers)."""
    return _struct_array(UpdateLayer, specs)


def fetch_layers(specs):
    """ctypes array of fg_fetch_layer_t from dicts keyed by the field names."""
    return _struct_array(FetchLayer, specs)


def fg_sample_block_workspace_bytes(max_rows, fanout):
    return int(_lib.fg_sample_block_workspace_bytes(max_rows, fanout))


def fg_sample_block(indptr, indices, num_nodes, num_edges, ids, n_dev, max_rows, fanout, key, layer, row_start, row_end, col, col_ids,
                    ids_below, max_below, counts, ws, ws_bytes, stream=None):
    _check(_lib.fg_sample_block(ptr(indptr), ptr(indices), num_nodes, num_edges, ptr(ids), ptr(n_dev), max_rows, fanout, key, layer,
                                ptr(row_start), ptr(row_end), ptr(col), ptr(col_ids), ptr(ids_below), max_below, ptr(counts),
                                ptr(ws), ws_bytes, stream))


def fg_transpose_block_workspace_bytes(max_src):
    return int(_lib.fg_transpose_block_workspace_bytes(max_src))


def fg_transpose_block(row_start, row_end, col, n_dev, max_rows, n_src_dev, max_src, max_nnz, t_start, t_end, t_row, ws, ws_bytes,
                       stream=None):
    _check(_lib.fg_transpose_block(ptr(row_start), ptr(row_end), ptr(col), ptr(n_dev), max_rows, ptr(n_src_dev), max_src, max_nnz,
                                   ptr(t_start), ptr(t_end), ptr(t_row), ptr(ws), ws_bytes, stream))


def fg_access_estimate(row_start, row_end, col, nnz, n, hit, below, n_src, out, stream=None):
    _check(_lib.fg_access_estimate(ptr(row_start), ptr(row_end), ptr(col), nnz, n, ptr(hit), ptr(below), n_src, ptr(out), stream))


def fg_cache_fetch_all(cache, layers, stream=None):
    _check(_lib.fg_cache_fetch_all(cache, len(layers), layers, stream))


def fg_cache_update_all(cache, it, p_grad, layers, ws, ws_bytes, stream=None):
    _check(_lib.fg_cache_update_all(cache, it, p_grad, len(layers), layers, ptr(ws), ws_bytes, stream))


def fg_cache_update_select(cache, it, p_grad, layers, ws, ws_bytes, stream=None):
    _check(_lib.fg_cache_update_select(cache, it, p_grad, len(layers), layers, ptr(ws), ws_bytes, stream))


def fg_cache_update_commit(cache, it, layers, ws, ws_bytes, stream=None):
    _check(_lib.fg_cache_update_commit(cache, it, len(layers), layers, ptr(ws), ws_bytes, stream))
