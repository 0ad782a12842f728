"""Pins of the oracle's feature side of the bidirectional cache (Section 4.2) against things that are not the
oracle: a byte-by-byte record of what the rings have written, the bit-identity of every loaded row with the
table, a hand-worked displacement trace, and order properties of the hot list. No GPU."""
import os

import numpy as np
import pytest

from fg_inputs.graph import ChungLuGraph
from oracle import freshgnn_oracle as O
from tests import helpers as T


def table_rows(num_nodes, dim, seed, dtype=np.float32):
    X = np.random.default_rng(seed).standard_normal((num_nodes, dim)).astype(dtype)
    return X, (lambda ids: X[np.asarray(ids, dtype=np.int64)])


def written_bytes(bc):
    """Every byte an embedding has been written to, from the slot owners alone (a slot that was ever written names a node)."""
    dirty = np.zeros(bc.buffer_bytes, dtype=bool)
    for l, ring in bc.rings.items():
        for s in range(ring.capacity):
            if ring.slot_node[s] >= 0:
                lo = bc.ring_base[l] + s * ring.row_bytes
                dirty[lo:lo + ring.row_bytes] = True
    return dirty


def drive_ring(ring, it, nodes, rng, p_grad=1.0):
    """One update of a ring with `nodes` as computed live nodes and random rows."""
    h = rng.standard_normal((len(nodes), ring.dim)).astype(np.float32)
    if ring.dtype == "bf16":
        h = O.round_bf16(h)
    g = np.exp(rng.standard_normal(len(nodes))).astype(np.float32)
    return O.cache_update(ring, it, np.asarray(nodes, dtype=np.int32), None, np.zeros(len(nodes), dtype=bool), g, p_grad, h), h


def test_trace_junction():
    params, hot, steps = {}, None, []
    for line in open(os.path.join(T.GOLDEN, "bidirectional_junction_trace.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("hot"):
            hot = [int(t) for t in line.split()[1:]]
        elif line.startswith("update"):
            f = [x.strip() for x in line.split("|")]
            steps.append((int(f[0].split()[1]), [int(t) for t in f[1].split()[1:]], [int(t) for t in f[2].split()[1:]]))
        else:
            k, v = line.split()
            params[k] = float(v) if "." in v else int(v)
    X, rows = table_rows(64, params["feat_dim"], 0)
    bc = O.BidirectionalCache(64, [params["capacity"]], [params["ring_dim"]], params["t_stale"], "f32", params["buffer_bytes"])
    bc.fill_features(hot, rows, "f32")
    assert [bc.feature_rank(v) for v in hot] == list(range(len(hot)))
    r = np.random.default_rng(1)
    for it, live, surviving in steps:
        drive_ring(bc.rings[1], it, live, r, params["p_grad"])
        assert [k for k, v in enumerate(hot) if bc.feature_rank(v) >= 0] == surviving, f"update {it}"


@pytest.mark.parametrize("seed,dtype,feat_dtype,buffer_bytes,caps,dims,feat_dim,n_hot", [
    (0, "f32", "f32", 4096, [5, 3], [12, 20], 8, 128),      # everything overlaps: the buffer starts full of features
    (1, "f32", "f32", 8192, [7, 4], [36, 8], 12, 170),      # rows of 144 / 32 bytes against feature rows of 48
    (2, "bf16", "f16", 4096, [9, 6], [24, 40], 24, 85),     # 16-bit storage on both sides
    (3, "f32", "f32", 3000 * 16, [40], [28], 4, 3000),      # one large ring, small rows
    (4, "f32", "f32", 2048, [3, 2, 2], [8, 8, 8], 8, 10),   # three rings, few features: only the right end is covered
])
def test_validity_equals_untouched_bytes_and_rows_stay_bit_identical(seed, dtype, feat_dtype, buffer_bytes, caps, dims, feat_dim, n_hot):
    N = 4000
    np_feat = np.float32 if feat_dtype == "f32" else np.float16
    X, rows = table_rows(N, feat_dim, seed, np_feat)
    r = np.random.default_rng(seed + 100)
    bc = O.BidirectionalCache(N, caps, dims, 4, dtype, buffer_bytes)
    hot = r.permutation(N)[:n_hot]
    bc.fill_features(hot, rows, feat_dtype)
    w = feat_dim * O.element_bytes(feat_dtype)
    next_node = 0
    seen_partial = False
    for it in range(12):
        # the check comes first, so the state before any update is covered too
        dirty = written_bytes(bc)
        for k, v in enumerate(hot):
            lo = buffer_bytes - (k + 1) * w
            untouched = not dirty[lo:lo + w].any()
            seen_partial |= bool(dirty[lo:lo + w].any() and not dirty[lo:lo + w].all())
            assert (bc.feature_rank(v) == k) == untouched, (it, k)
            assert bc.feature_rank(v) in (k, -1)
        ids = r.permutation(N)[:300]
        got, from_buffer = bc.load(ids, rows)
        assert got.dtype == X.dtype and np.array_equal(got.view(np.uint8), X[ids].view(np.uint8))
        assert np.array_equal(from_buffer, np.asarray([bc.feature_rank(v) >= 0 for v in ids]))
        assert not from_buffer[~np.isin(ids, hot)].any()
        for l, ring in bc.rings.items():   # uneven admission counts; some updates admit nothing
            n_new = int(r.integers(0, 3))
            nodes = np.arange(next_node, next_node + n_new)
            next_node += n_new
            if n_new:
                drive_ring(ring, it, nodes, r)
    assert all(ring.used == min(ring.capacity, int((ring.slot_node >= 0).sum())) for ring in bc.rings.values())
    if seed in (0, 1, 2):
        assert seen_partial, "the case was meant to contain a feature row cut by the end of a written slot"


def test_ring_rows_are_laid_down_in_the_shared_buffer():
    N = 100
    X, rows = table_rows(N, 8, 0)
    for dtype in ("f32", "bf16"):
        bc = O.BidirectionalCache(N, [4, 3], [8, 16], 5, dtype, 2048)
        bc.fill_features(np.arange(20), rows, "f32")
        r = np.random.default_rng(3)
        _, h1 = drive_ring(bc.rings[1], 0, [50, 51, 52], r)
        _, h2 = drive_ring(bc.rings[2], 0, [60], r)
        es = O.element_bytes(dtype)
        assert bc.ring_base == {1: 0, 2: 256}      # 4 * 8 * es <= 256: the second ring starts at the alignment
        for ring, base, h in ((bc.rings[1], 0, h1), (bc.rings[2], 256, h2)):
            for s in range(len(h)):
                raw = bc.buf[base + s * ring.row_bytes: base + (s + 1) * ring.row_bytes]
                if dtype == "f32":
                    assert np.array_equal(raw.view(np.float32), h[s])
                else:
                    assert np.array_equal((raw.view(np.uint16).astype(np.uint32) << 16).view(np.float32), h[s])
                assert es * ring.dim == ring.row_bytes


def test_one_ring_keeps_a_prefix_of_the_hot_list():
    """With a single ring the surviving rows are always the hottest ones: rank r survives only if every rank below it does."""
    N = 500
    X, rows = table_rows(N, 4, 0)
    bc = O.BidirectionalCache(N, [30], [12], 3, "f32", 30 * 48 + 160)
    hot = np.random.default_rng(0).permutation(N)[:(30 * 48 + 160) // 16]
    bc.fill_features(hot, rows, "f32")
    r = np.random.default_rng(1)
    survivors = []
    for it in range(20):
        drive_ring(bc.rings[1], it, np.arange(it * 2, it * 2 + 2), r)
        alive = np.asarray([bc.feature_rank(v) >= 0 for v in hot])
        k = int(alive.sum())
        assert alive[:k].all() and not alive[k:].any()
        survivors.append(k)
    assert survivors == sorted(survivors, reverse=True) and survivors[0] < len(hot)
    assert survivors[-1] == 160 // 16        # what lies beyond the ring stays for good


def test_hot_order_properties():
    r = np.random.default_rng(0)
    score = r.integers(0, 6, size=200).astype(np.float64)   # many ties
    for count in (0, 1, 37, 200):
        order = O.hot_order(score, count)
        assert len(order) == count and len(set(order.tolist())) == count
        s = score[order]
        assert np.all(s[:-1] >= s[1:])
        same = s[:-1] == s[1:]
        assert np.all(order[:-1][same] < order[1:][same])
        left_out = np.setdiff1d(np.arange(200), order)
        if count and len(left_out):
            assert score[left_out].max() <= s[-1]
            at_edge = left_out[score[left_out] == s[-1]]
            assert len(at_edge) == 0 or at_edge.min() > order[s == s[-1]].max()


def test_generated_graph_lists_its_hottest_nodes_in_that_order():
    g = ChungLuGraph(5000, 60000, 3)
    score = g.access_estimate(np.arange(5000))
    assert np.array_equal(g.hottest(400), O.hot_order(score, 400))
    ex = T.random_explicit_graph(80, 6, 1)
    assert ex.access_estimate().sum() == len(ex.indices)


def run_with_feature_side(use_feature_side, buffer_bytes=1 << 14, n_iter=8):
    """A cached 3-layer run on a small graph; returns per-iteration records."""
    g = T.random_explicit_graph(300, 6, 4, allow_isolated=False)
    dims = [8, 12, 12, 5]
    X, rows = table_rows(300, 8, 5)
    weights = T.random_weights(dims, 6)
    bc = O.BidirectionalCache(300, [40, 30], [12, 12], 3, "f32", buffer_bytes)
    if use_feature_side:
        bc.fill_features(O.hot_order(g.access_estimate(), buffer_bytes // 32), rows, "f32")
    recs = []
    for it in range(n_iter):
        seeds = np.random.default_rng(50 + it).permutation(300)[:12]
        mb = T.sample(g, seeds, [4, 4, 4], it)
        r = np.random.default_rng(900 + it)
        gn = {l: np.exp(r.standard_normal(len(mb.ids[l]))).astype(np.float32) for l in (1, 2)}
        recs.append(O.iteration(mb, it, bc.rings, rows, weights, gn, 0.6, dims, feature_side=bc if use_feature_side else None))
    return recs, bc


def test_feature_side_changes_where_rows_come_from_and_nothing_else():
    with_fs, bc = run_with_feature_side(True)
    without, _ = run_with_feature_side(False)
    served = []
    for a, b in zip(with_fs, without):
        for l in range(4):
            assert np.array_equal(a["H"][l].view(np.uint8), b["H"][l].view(np.uint8))
        assert a["stats"] == b["stats"]
        assert len(a["feature_from_buffer"]) == len(a["look"][0]["normal_pos"])
        assert not b["feature_from_buffer"].any()
        served.append(int(a["feature_from_buffer"].sum()))
    assert served[0] > 0
    # the rings fill and push the feature side back: fewer rows are served from the buffer at the end than at the start
    assert all(r.used > 0 for r in bc.rings.values())
    assert served[-1] < served[0]
