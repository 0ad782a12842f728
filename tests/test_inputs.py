"""The synthetic input generators: determinism, layout, distribution shape (no GPU)."""
import numpy as np

from fg_inputs import features, rng, workload as wl
from fg_inputs.graph import ChungLuGraph
from oracle.freshgnn_oracle import check_minibatch


def test_splitmix64_published_vector():
    # first outputs of SplitMix64 seeded with 0 (state advances by GAMMA before each output)
    assert int(rng.mix64(rng.GAMMA)) == 0xE220A8397B1DCDAF
    assert int(rng.u64(np.uint64(0), 1)) == 0x6E789E6AA1B965F4


def test_features_are_a_pure_function_of_seed_node_column():
    a = features.feature_rows(5, [7, 3, 7, 10 ** 8], 16)
    b = features.feature_rows(5, [3], 16)
    assert np.array_equal(a[0], a[2]) and np.array_equal(a[1], b[0]) and not np.array_equal(a[0], a[1])
    big = features.feature_rows(5, np.arange(4000), 64)
    assert abs(big.mean()) < 0.01 and abs(big.std() - 1.0) < 0.01
    h = features.feature_rows(5, [3], 16, np.float16)
    assert np.array_equal(h, b.astype(np.float16))


def test_chung_lu_degrees_and_bijection():
    g = ChungLuGraph(100_000, 1_000_000, seed=1)
    v = np.arange(100_000)
    assert np.array_equal(np.sort(g.rank_to_id(v)), v)
    assert np.array_equal(g.id_to_rank(g.rank_to_id(v)), v)
    d = g.degree(v)
    assert abs(d.mean() - 10.0) < 0.2 and d.max() > 50 * d.mean()          # heavy tail
    assert np.array_equal(d, g.degree(v))
    nb = g.neighbour(np.full(20000, 17), np.arange(20000))
    assert nb.min() >= 0 and nb.max() < 100_000
    # neighbours are drawn in proportion to expected degree: hubs (low rank) dominate
    assert (g.id_to_rank(nb) < 1000).mean() > 0.05


def test_minibatch_layout_and_determinism():
    w = wl.WORKLOADS["tiny"]
    g = wl.make_graph(w)
    a, b = wl.minibatch(w, g, 3), wl.minibatch(w, g, 3)
    check_minibatch(a)
    for l in range(w.num_layers + 1):
        assert np.array_equal(a.ids[l], b.ids[l]) and a.ids[l].dtype == np.int32
    for l in range(1, w.num_layers + 1):
        assert np.array_equal(a.col[l], b.col[l])
        deg = a.end[l] - a.start[l]
        assert deg.max() <= w.fanouts[l - 1]
        for j in range(0, len(deg), 37):                       # no self loops, no repeats within a row
            nb = a.col[l][a.start[l][j]:a.end[l][j]]
            assert j not in nb and len(set(nb.tolist())) == len(nb)
    c = wl.minibatch(w, g, 4)
    assert not np.array_equal(a.ids[w.num_layers], c.ids[w.num_layers])
    assert len(np.unique(wl.seed_nodes(w, 0))) == w.batch


def test_grad_norms_and_weights():
    w = wl.WORKLOADS["tiny"]
    gn = wl.grad_norms(w, 2, 1, np.arange(20000))
    assert gn.dtype == np.float32 and gn.min() > 0 and abs(np.log(gn).std() - 1.0) < 0.05
    assert np.array_equal(gn[:5], wl.grad_norms(w, 2, 1, np.arange(5)))
    W, b = wl.layer_weights(w, 1)
    assert W.shape == (128, 64) and b.shape == (64,) and abs(W.std() - 1 / np.sqrt(128)) < 0.01


def test_transposed_block_lists_the_rows_that_sampled_each_position():
    from fg_inputs.sampler import transpose_block
    from tests import helpers as T
    g = T.random_explicit_graph(50, 5, 0)
    mb = T.sample(g, np.arange(8), [3, 3], 0)
    for l in (1, 2):
        ts, te, tr = transpose_block(mb.start[l], mb.end[l], mb.col[l], len(mb.ids[l - 1]))
        for j in range(len(mb.ids[l - 1])):
            want = [r for r in range(len(mb.ids[l])) if j in mb.col[l][mb.start[l][r]:mb.end[l][r]]]
            assert tr[ts[j]:te[j]].tolist() == want
        assert te[-1] == len(tr) == int((mb.end[l] - mb.start[l]).sum())
