"""The C-ABI library: loads, exports everything the header declares, and rejects bad arguments on the host
before anything is launched (so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "freshgnn.h")


@pytest.fixture(scope="module")
def B():
    from paper_2301_07482_amd import binding
    return binding


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fg_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(B):
    names = declared_functions()
    assert {"fg_cache_create", "fg_lookup_prune", "fg_gather", "fg_aggregate", "fg_linear", "fg_cache_update"} <= set(names)
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in freshgnn.h but not exported"
    assert set(B.SIGNATURES) == set(names), "binding and header list different calls"
    assert B.fg_version() >= 100


def test_argument_validation_needs_no_gpu(B):
    def code(fn, *a, **k):
        with pytest.raises(B.FgError) as e:
            fn(*a, **k)
        assert B.fg_last_error() != ""
        return e.value.code

    assert code(B.fg_gather, None, 10, 16, 16, None, None, None, 4, None, 4, 16) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_gather, 4096, 10, 16, 15, 4096, None, None, 4, 4096, 4, 16) == B.FG_ERR_SHAPE          # odd row
    assert code(B.fg_gather, 4096, 10, 8, 16, 4096, None, None, 4, 4096, 4, 16) == B.FG_ERR_SHAPE           # stride < row
    assert code(B.fg_gather, 4100, 10, 16, 16, 4096, None, None, 4, 4096, 4, 16) == B.FG_ERR_INVALID_ARG    # alignment
    assert code(B.fg_gather, 4096, 10, 16, 16, 4096, None, None, -1, 4096, 4, 16) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_gather, 4096, 10, 16, 16, 4096, None, None, 4, 4096, 4, 16, 7) == B.FG_ERR_INVALID_ARG  # table kind
    assert code(B.fg_lookup_prune, None, 0, 0, None, 5, None, None, None, None, 0, 0, None, None, None, None, None, None,
                None, None, 0) == B.FG_ERR_INVALID_ARG                                                      # no counts
    assert code(B.fg_lookup_prune, None, 0, 0, 4096, 5, None, 4096, None, None, 0, 9, None, None, None, None, 4096, None,
                4096, None, 0) == B.FG_ERR_INVALID_ARG                                                      # half a block
    assert code(B.fg_lookup_prune, None, 0, 0, 4096, 5, None, 4096, 4096, 4096, 3, 2, 4096, None, None, None, 4096, None,
                4096, 4096, 1 << 20) == B.FG_ERR_SHAPE                                                      # n_src < n
    assert code(B.fg_lookup_prune, None, 0, 0, 4096, 5, None, None, None, None, 0, 0, None, None, None, None, 4096, None,
                4096, 4096, 8) == B.FG_ERR_SHAPE                                                            # workspace
    assert code(B.fg_aggregate, 4096, 4096, 4096, 5, 5, None, None, 5, 4096, 9, 512, 130, B.FG_F32, 4096, 520, B.FG_F32) \
        == B.FG_ERR_SHAPE                                                                                   # dim % 4
    assert code(B.fg_aggregate, 4096, 4096, 4096, 5, 5, None, None, 5, 4096, 9, 256, 128, B.FG_F32, 4096, 512, B.FG_F32) \
        == B.FG_ERR_SHAPE                                                                                   # stride
    assert code(B.fg_aggregate, 4096, 4096, 4096, 5, 5, None, None, 5, 4096, 9, 512, 128, 9, 4096, 512, B.FG_F32) \
        == B.FG_ERR_DTYPE
    assert code(B.fg_linear, 4096, 9, 512, B.FG_F32, 4096, 512, None, None, 5, 126, 64, 4096, B.FG_F32, None, 1, 4096, 9, 256,
                B.FG_F32) == B.FG_ERR_SHAPE
    assert code(B.fg_linear, 4096, 9, 512, B.FG_F16, 4096, 512, None, None, 5, 128, 64, 4096, B.FG_F32, None, 1, 4096, 9, 256,
                B.FG_F32) == B.FG_ERR_DTYPE
    assert code(B.fg_linear, None, 9, 512, B.FG_F32, 4096, 512, None, None, 5, 128, 64, 4096, B.FG_F32, None, 1, 4096, 9, 256,
                B.FG_F32) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_update, None, 1, 0, None, 0, None, None, None, 0.5, None, 0, None, None, 0) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_update_all, None, 0, 0.5, B.update_layers([dict(layer=1, n=0)]), None, 0) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_update_all, None, 0, 0.5, B.update_layers([dict(layer=1, n=0)] * 9), None, 0) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_update_select, None, 0, 0.5, B.update_layers([dict(layer=1, n=0)]), None, 0) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_update_commit, None, 0, B.update_layers([dict(layer=1, n=0)]), None, 0) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_fetch_all, None, B.fetch_layers([dict(layer=1)])) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_fetch_all, None, B.fetch_layers([dict(layer=1)] * 9)) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_create, 0, [4], [4], B.FG_F32, 3) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_create, 100, [0], [4], B.FG_F32, 3) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_create, 100, [4], [3], B.FG_F32, 3) == B.FG_ERR_SHAPE
    assert code(B.fg_cache_create, 100, [4], [4], 5, 3) == B.FG_ERR_DTYPE
    assert code(B.fg_cache_create, 100, [4], [4], B.FG_F32, -1) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_create_bidirectional, 100, [4], [4], B.FG_F32, 3, 0) == B.FG_ERR_INVALID_ARG        # no buffer
    assert code(B.fg_cache_create_bidirectional, 100, [4], [4], B.FG_F32, 3, 1000) == B.FG_ERR_INVALID_ARG     # not a multiple of 256
    assert code(B.fg_cache_create_bidirectional, 100, [100], [64], B.FG_F32, 3, 1024) == B.FG_ERR_SHAPE        # rings do not fit
    assert code(B.fg_cache_create_bidirectional, 100, [4] * 9, [4] * 9, B.FG_F32, 3, 1 << 20) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_cache_fill_features, None, 4096, 4, 4096, 10, 64, 64) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_feature_lookup, None, 4096, None, 4, 4096, None) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_gather_features, None, 4096, 10, 16, 16, 4096, None, None, 4, 4096, 4, 16) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_gather_aggregate_features, None, 4096, 4096, 4096, 5, 5, None, None, 5, 4096, 9, 4096, 9, 512, 128, B.FG_F32,
                4096, 512, B.FG_F32) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_gather_aggregate_ids, 4096, 4096, 4096, 5, 5, None, None, 5, None, 4096, 9, 512, 128, B.FG_F32, 4096, 512,
                B.FG_F32) == B.FG_ERR_INVALID_ARG                                                           # no row ids
    assert code(B.fg_gather_aggregate_ids, 4096, 4096, 4096, 5, 5, None, None, 5, 4096, 4096, 9, 512, 128, B.FG_F32, 4096, 512,
                B.FG_F32, cache=None, fetch_layers=B.fetch_layers([dict(layer=1)])) == B.FG_ERR_INVALID_ARG # a fetch needs a cache
    assert code(B.fg_access_estimate, None, 4096, 4096, 5, 5, None, None, 9, 4096) == B.FG_ERR_INVALID_ARG         # no row starts
    assert code(B.fg_access_estimate, 4096, 4096, 4096, 5, 5, None, 4096, 3, 4096) == B.FG_ERR_SHAPE             # layer below smaller
    assert code(B.fg_access_estimate, 4096, 4096, 4096, 5, -1, None, None, 9, 4096) == B.FG_ERR_INVALID_ARG
    smp = lambda **k: B.fg_sample_block(**{**dict(indptr=4096, indices=4096, num_nodes=100, num_edges=500, ids=4096, n_dev=None, max_rows=10,
                                                  fanout=5, key=7, layer=1, row_start=4096, row_end=4096, col=4096, col_ids=None,
                                                  ids_below=4096, max_below=60, counts=4096, ws=4096, ws_bytes=1 << 30), **k})
    assert code(smp, fanout=33) == B.FG_ERR_INVALID_ARG and code(smp, fanout=0) == B.FG_ERR_INVALID_ARG
    assert code(smp, layer=0) == B.FG_ERR_INVALID_ARG and code(smp, counts=None) == B.FG_ERR_INVALID_ARG
    assert code(smp, max_below=9) == B.FG_ERR_SHAPE and code(smp, ws_bytes=64) == B.FG_ERR_SHAPE
    assert code(smp, ids=None) == B.FG_ERR_INVALID_ARG and code(smp, num_nodes=1 << 31) == B.FG_ERR_INVALID_ARG
    assert B.fg_sample_block_workspace_bytes(1000, 15) >= 1000 * 15 * 16 and B.fg_sample_block_workspace_bytes(10, 40) == 0
    assert code(B.fg_transpose_block, None, 4096, 4096, None, 10, None, 30, 50, 4096, 4096, 4096, 4096, 1 << 20) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_transpose_block, 4096, 4096, 4096, None, 10, None, 30, 50, 4096, 4096, None, 4096, 1 << 20) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_transpose_block, 4096, 4096, 4096, None, 10, None, 30, 50, 4096, 4096, 4096, 4096, 16) == B.FG_ERR_SHAPE
    assert B.fg_transpose_block_workspace_bytes(5000) >= 5000 * 4 and B.fg_transpose_block_workspace_bytes(-1) == 0
    assert B.fg_cache_feature_rows(None) == 0 and B.fg_cache_buffer(None) == (None, 0) and B.fg_cache_ring_offset(None, 1) == -1
    assert code(B.fg_softmax_xent_grad, None, 64, 4096, 4, 16, 4096, 64) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_softmax_xent_grad, 4096, 32, 4096, 4, 16, 4096, 64) == B.FG_ERR_SHAPE                     # stride < row
    assert code(B.fg_row_norms, 4096, 64, 4, 0, 4096) == B.FG_ERR_INVALID_ARG
    bw = lambda **k: B.fg_layer_backward(**{**dict(dh=4096, dh_stride=1024, h=4096, h_stride=1024, n=10, rows=4096, n_rows=None,
                                                   max_rows=10, live=None, hit=None, row_start=4096, row_end=4096, t_start=4096,
                                                   t_end=4096, t_row=4096, nnz=50, n_src=30, d_in=128, d_out=256, W=4096,
                                                   dh_src=4096, dh_src_stride=512, norms_src=None, ws=4096, ws_bytes=1 << 30), **k})
    assert code(bw, n_src=5) == B.FG_ERR_SHAPE              # the layer below is smaller
    assert code(bw, max_rows=11) == B.FG_ERR_SHAPE
    assert code(bw, d_out=252) == B.FG_ERR_SHAPE
    assert code(bw, ws_bytes=100) == B.FG_ERR_SHAPE
    assert code(bw, dh_src=None) == B.FG_ERR_INVALID_ARG
    assert code(bw, dh_src_stride=500) == B.FG_ERR_SHAPE
    assert B.fg_layer_backward_workspace_bytes(10, 10, 128, 256) >= 10 * (256 * 4 + 2 * 128 * 4) + 2 * 128 * 256 * 4
    assert B.fg_layer_backward_workspace_bytes(-1, 10, 128, 256) == 0
    assert code(B.fg_layer_backward_weights, 4096, 10, 512, 4096, 512, 4096, 1024, None, 0, 10, 4096, None, 10, 128, 256, None, None,
                4096, 1 << 30) == B.FG_ERR_INVALID_ARG                                                      # no dw
    assert code(B.fg_layer_backward_weights, 4096, 10, 512, 4096, 512, 4096, 1024, None, 0, 10, 4096, None, 10, 128, 256, 4096, None,
                4096, 64) == B.FG_ERR_SHAPE                                                                 # workspace
    assert B.fg_layer_backward_weights_workspace_bytes(67584, 128, 256) >= 256 * 256 * 4
    # GCN and mixed-precision forms of the layer backward: the same argument list, their own shape rules
    assert code(bw, kind="gcn", n_src=5) == B.FG_ERR_SHAPE and code(bw, kind="gcn", dh_src_stride=500) == B.FG_ERR_SHAPE
    assert code(bw, kind="gcn", ws_bytes=100) == B.FG_ERR_SHAPE
    assert code(bw, kind="bf16", d_out=248) == B.FG_ERR_SHAPE           # d_out % 16
    assert code(bw, kind="bf16", d_in=132) == B.FG_ERR_SHAPE            # d_in % 8
    assert code(bw, kind="bf16", W=4100) == B.FG_ERR_INVALID_ARG        # W 16-byte aligned
    assert code(bw, kind="bf16", h_stride=256) == B.FG_ERR_SHAPE        # bf16 rows of 256 values need 512 bytes
    assert B.fg_layer_backward_workspace_bytes(10, 10, 128, 256, kind="gcn") < B.fg_layer_backward_workspace_bytes(10, 10, 128, 256)
    assert B.fg_layer_backward_workspace_bytes(10, 10, 128, 256, kind="bf16") < B.fg_layer_backward_workspace_bytes(10, 10, 128, 256)
    assert B.fg_layer_backward_workspace_bytes(10, 10, 128, 256, kind="bf16") >= 10 * 2 * 128 * 4 + 10 * 256 * 2
    wg16 = lambda **k: B.fg_layer_backward_weights_bf16(**{**dict(h_src=4096, n_src=10, src_stride=256, src_dtype=B.FG_BF16, agg=4096,
                                                                   agg_stride=256, dh=4096, dh_stride=1024, h=None, h_stride=0, n=10,
                                                                   rows=4096, n_rows=None, max_rows=10, d_in=128, d_out=256, dw=4096,
                                                                   db=None, ws=4096, ws_bytes=1 << 30), **k})
    assert code(wg16, dw=None) == B.FG_ERR_INVALID_ARG and code(wg16, ws_bytes=64) == B.FG_ERR_SHAPE
    assert code(wg16, src_dtype=9) == B.FG_ERR_DTYPE and code(wg16, d_in=132) == B.FG_ERR_SHAPE
    assert code(wg16, src_dtype=B.FG_F32) == B.FG_ERR_SHAPE             # fp32 rows of 128 values need a stride of 512 bytes
    lin_wt = lambda **k: B.fg_linear_wt(**{**dict(h_src=4096, n_src=9, src_stride=256, in_dtype=B.FG_BF16, agg=4096, agg_stride=256,
                                                   rows=None, n_rows=None, max_rows=5, d_in=128, d_out=64, Wt=4096, w_dtype=B.FG_BF16,
                                                   bias=None, relu=1, h_out=4096, n_out=9, out_stride=128, out_dtype=B.FG_BF16), **k})
    assert code(lin_wt, w_dtype=B.FG_F32) == B.FG_ERR_DTYPE             # transposed weights are taken in bf16 only
    assert code(lin_wt, Wt=None) == B.FG_ERR_INVALID_ARG and code(lin_wt, d_in=124) == B.FG_ERR_SHAPE
    assert code(lin_wt, in_dtype=B.FG_F32) == B.FG_ERR_DTYPE and code(lin_wt, out_stride=64) == B.FG_ERR_SHAPE
    lin_ids = lambda **k: B.fg_linear_ids(**{**dict(table=4096, table_rows=90, src_stride=512, in_dtype=B.FG_F32, src_ids=4096,
                                                     agg=4096, agg_stride=512, rows=None, n_rows=None, max_rows=5, d_in=128, d_out=64,
                                                     W=4096, w_dtype=B.FG_F32, bias=None, relu=1, h_out=4096, n_out=9,
                                                     out_stride=256, out_dtype=B.FG_F32), **k})
    assert code(lin_ids, src_ids=None) == B.FG_ERR_INVALID_ARG and code(lin_ids, table=None) == B.FG_ERR_INVALID_ARG
    assert code(lin_ids, src_stride=256) == B.FG_ERR_SHAPE and code(lin_ids, in_dtype=B.FG_F16) == B.FG_ERR_DTYPE
    assert code(lin_ids, table_rows=-1) == B.FG_ERR_INVALID_ARG
    lin_ids(max_rows=0, src_ids=None)                                   # nothing to do: no launch, no error
    # the allocation-free lookup refuses what its built-in scratch memory cannot hold
    assert code(B.fg_lookup_prune_static, None, 0, 0, 4096, B.FG_LOOKUP_PRUNE_STATIC_MAX_N + 1, None, None, None, None, 0, 0, None, None,
                None, None, 4096, None, 4096) == B.FG_ERR_SHAPE
    assert code(B.fg_cache_set_stabilization, None, 3) == B.FG_ERR_INVALID_ARG
    assert code(B.fg_aggregate_linear, 4096, 4096, 4096, 5, 5, None, None, 5, None, 9, 512, 128, 64, 4096, None, 0, None, 512, 4096, 5,
                256) == B.FG_ERR_INVALID_ARG                                                                # no h_src
    assert code(B.fg_aggregate_linear, 4096, 4096, 4096, 5, 50000, None, None, 50000, 4096, 50000, 512, 128, 64, 4096, None, 0, None,
                512, 4096, 50000, 256) == B.FG_ERR_INVALID_ARG                                              # two launches need agg_ws
    assert B.one_launch_layer(1024, 256, 256) and not B.one_launch_layer(6144, 256, 256) and not B.one_launch_layer(100, 100, 64)
    assert code(B.fg_set_tuning, "gather_unroll", -3) == B.FG_ERR_INVALID_ARG
    assert B.fg_workspace_bytes(B.FG_WS_LOOKUP_PRUNE, 1000) >= 1000 * 5
    assert B.fg_workspace_bytes(B.FG_WS_CACHE_UPDATE, 1000) >= 1000 * 9
    assert B.fg_workspace_bytes(7, 1000) == 0


def test_zero_sized_calls_are_noops_without_gpu(B):
    B.fg_gather(None, 0, 16, 16, None, None, None, 0, None, 0, 16)
    B.fg_aggregate(None, None, None, 0, 0, None, None, 0, None, 0, 16, 4, B.FG_F32, None, 16, B.FG_F32)
    B.fg_cache_destroy(None)


def test_header_is_plain_c(tmp_path):
    """include/freshgnn.h compiles as C99 and as C++17 on its own (no torch or HIP types in the boundary)."""
    import shutil
    import subprocess
    src = tmp_path / "uses_header.c"
    src.write_text('#include "freshgnn.h"\nint main(void) { return 0; }\n')
    inc = os.path.join(ROOT, "include")
    for cc, std in (("gcc", "-std=c99"), ("g++", "-std=c++17")):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not found")
        args = [cc, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-fsyntax-only"] + (["-x", "c++"] if cc == "g++" else []) + [str(src)]
        p = subprocess.run(args, capture_output=True, text=True)
        assert p.returncode == 0, p.stderr


def test_three_way_bf16_split_is_exact_on_the_documented_input_domain():
    """fg_linear forms fp32 products from an exact three-way bf16 split of both factors (x = x1 + x2 + x3, each term the
    bf16 nearest to what is left). A host model of that split, with bf16 subnormals flushed to zero as the matrix
    instructions may do: it loses nothing for magnitudes in [2^-100, 2^127), which is the domain the header documents,
    and it does lose bits once the third term falls below the smallest normal bf16 (magnitudes near 2^-112 and below)."""
    import numpy as np

    def bf16_flush(x):
        x = x.astype(np.float32)
        b = x.view(np.uint32).astype(np.uint64)
        r = ((b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000).astype(np.uint32).view(np.float32)
        return np.where(np.abs(r) < np.float32(2.0 ** -126), np.float32(0), r)

    def split_error(x):
        x1 = bf16_flush(x)
        r1 = (x - x1).astype(np.float32)
        x2 = bf16_flush(r1)
        r2 = (r1 - x2).astype(np.float32)
        x3 = bf16_flush(r2)
        return np.abs(x.astype(np.float64) - (x1.astype(np.float64) + x2.astype(np.float64) + x3.astype(np.float64))) / np.abs(x)

    r = np.random.default_rng(0)
    mant = (1.0 + r.random(200000)).astype(np.float32) * np.where(r.random(200000) < 0.5, -1, 1).astype(np.float32)
    for e in (-100, -60, 0, 60, 126):
        x = (mant * np.float32(2.0 ** e)).astype(np.float32)
        assert split_error(x).max() == 0.0, e
    assert split_error((mant * np.float32(2.0 ** -114)).astype(np.float32)).max() > 2.0 ** -20
