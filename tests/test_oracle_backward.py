"""Pins of the oracle's loss and backward pass (Alg. 1, loss / loss.backward(); Section 4.1.1) against central finite
differences of the loss through the oracle's forward functions, and against closed forms. No GPU."""
import numpy as np
import pytest

from oracle import freshgnn_oracle as O
from tests import helpers as T


def forward_from(mb, rec, weights, l0, H_l0, W_override=None):
    """Loss as a function of H(l0) (and optionally of the weights of the layers above): layers l0+1..L recomputed in
    float64 on the pruned blocks of `rec`, fetched rows kept as the constants they are."""
    L = mb.num_layers
    H = np.asarray(H_l0, dtype=np.float64)
    for l in range(l0 + 1, L + 1):
        rows = rec["look"][l]["normal_pos"]
        W, b = (W_override or weights)[l]
        out = np.asarray(rec["H"][l], dtype=np.float64).copy()      # fetched (and dead) rows stay what they were
        agg = O.aggregate(mb.start[l], mb.end[l], mb.col[l], rows, H)
        out[rows] = O.linear(H[rows], agg, W, b, relu=(l < L))
        H = out
    return H


def cached_run(L=3, n_iter=5, seed=0):
    """A few iterations with an active cache on a small graph; returns the last iteration's record with its inputs."""
    g = T.random_explicit_graph(120, 5, seed, allow_isolated=True)
    dims = [6, 7, 8, 5][:L + 1]
    X = np.random.default_rng(seed).standard_normal((120, dims[0])).astype(np.float32)
    weights = T.random_weights(dims, seed + 1)
    caches = {l: O.HistoricalCache(120, 60, dims[l], 3) for l in range(1, L)}
    r = np.random.default_rng(seed + 2)
    for it in range(n_iter):
        seeds = r.permutation(120)[:10]
        labels = r.integers(0, dims[L], size=10)
        mb = T.sample(g, seeds, [3] * L, it)
        rec = O.iteration(mb, it, caches, lambda ids: X[ids], weights, None, 0.7, dims, labels=labels)
    return mb, rec, weights, labels, dims


def test_loss_gradient_against_finite_differences_and_row_sums():
    r = np.random.default_rng(0)
    h = r.standard_normal((7, 9)) * 3
    y = r.integers(0, 9, size=7)
    g = O.softmax_xent_grad(h, y)
    assert np.allclose(g.sum(axis=1), 0, atol=1e-15)           # softmax sums to one
    assert np.all(g[np.arange(7), y] < 0) and np.all(np.delete(g, y[0], axis=1)[0] > 0)
    eps = 1e-6
    for i, c in [(0, 0), (3, int(y[3])), (6, 8), (2, 5)]:
        hp, hm = h.copy(), h.copy()
        hp[i, c] += eps
        hm[i, c] -= eps
        assert abs((O.softmax_xent(hp, y) - O.softmax_xent(hm, y)) / (2 * eps) - g[i, c]) < 1e-8
    # uniform logits: loss = log(d), gradient = (1/d - onehot)/n
    u = np.zeros((4, 5))
    assert abs(O.softmax_xent(u, [0, 1, 2, 3]) - np.log(5)) < 1e-12
    assert np.allclose(O.softmax_xent_grad(u, [0, 1, 2, 3])[1], (np.full(5, 0.2) - np.eye(5)[1]) / 4)


def test_row_norms():
    x = np.random.default_rng(1).standard_normal((11, 6))
    assert np.allclose(O.row_norms(x), np.linalg.norm(x, axis=1), rtol=1e-14)
    assert O.row_norms(np.zeros((3, 4))).tolist() == [0, 0, 0]
    assert np.allclose(O.row_norms([[3.0, 4.0]]), [5.0])


@pytest.mark.parametrize("L,seed", [(2, 0), (3, 1), (3, 2)])
def test_embedding_gradients_against_finite_differences(L, seed):
    mb, rec, weights, labels, dims = cached_run(L=L, seed=seed)
    bw = rec["backward"]
    assert sum(len(rec["look"][l]["hit_pos"]) for l in range(1, L)) > 0, "the case was meant to contain fetched rows"
    loss = lambda l, H: O.softmax_xent(forward_from(mb, rec, weights, l, H), labels)
    eps = 1e-5
    r = np.random.default_rng(seed)
    for l in range(1, L + 1):
        base = np.asarray(rec["H"][l], dtype=np.float64)
        assert abs(loss(l, base) - O.softmax_xent(rec["H"][L], labels)) < 1e-5      # the test's forward reproduces the record
        live = rec["live"][l] if rec["live"][l] is not None else np.ones(len(base), bool)
        picks = [(int(j), int(c)) for j in r.permutation(len(base))[:12] for c in r.permutation(dims[l])[:2]]
        for j, c in picks:
            hp, hm = base.copy(), base.copy()
            hp[j, c] += eps
            hm[j, c] -= eps
            num = (loss(l, hp) - loss(l, hm)) / (2 * eps)
            assert abs(num - bw["dH"][l][j, c]) < 1e-7 + 1e-4 * abs(num), (l, j, c)
        # pruned positions receive nothing; fetched rows do receive their gradient
        assert not bw["dH"][l][~live].any()
        hp_ = rec["look"][l]["hit_pos"] if l < L else []
        if len(hp_):
            assert np.abs(bw["dH"][l][hp_]).sum() > 0
    for l in range(1, L):
        assert bw["gnorm"][l].dtype == np.float32
        assert np.allclose(bw["gnorm"][l], np.linalg.norm(bw["dH"][l], axis=1), rtol=1e-6)


def test_weight_gradients_against_finite_differences():
    mb, rec, weights, labels, dims = cached_run(L=3, seed=4)
    bw = rec["backward"]
    eps = 1e-5
    r = np.random.default_rng(0)
    for l in (1, 2, 3):
        W, b = weights[l]
        base_prev = np.asarray(rec["H"][l - 1], dtype=np.float64)
        for _ in range(6):
            a, c = int(r.integers(0, W.shape[0])), int(r.integers(0, W.shape[1]))
            out = []
            for sgn in (+1, -1):
                W2 = W.astype(np.float64).copy()
                W2[a, c] += sgn * eps
                ws = dict(weights)
                ws[l] = (W2, b)
                out.append(O.softmax_xent(forward_from(mb, rec, weights, l - 1, base_prev, W_override=ws), labels))
            num = (out[0] - out[1]) / (2 * eps)
            assert abs(num - bw["dW"][l][a, c]) < 1e-7 + 1e-4 * abs(num), (l, a, c)
        c = int(r.integers(0, len(b)))
        out = []
        for sgn in (+1, -1):
            b2 = b.astype(np.float64).copy()
            b2[c] += sgn * eps
            ws = dict(weights)
            ws[l] = (W, b2)
            out.append(O.softmax_xent(forward_from(mb, rec, weights, l - 1, base_prev, W_override=ws), labels))
        assert abs((out[0] - out[1]) / (2 * eps) - bw["db"][l][c]) < 1e-7


def test_gradient_norms_from_the_backward_pass_drive_the_update():
    """`iteration(labels=...)` admits by the norms of its own backward pass: the same update as passing those norms in."""
    g = T.random_explicit_graph(100, 5, 3)
    dims = [6, 7, 5]
    X = np.random.default_rng(0).standard_normal((100, 6)).astype(np.float32)
    weights = T.random_weights(dims, 1)
    ca = {1: O.HistoricalCache(100, 50, 7, 3)}
    cb = {1: O.HistoricalCache(100, 50, 7, 3)}
    r = np.random.default_rng(2)
    for it in range(5):
        seeds = r.permutation(100)[:8]
        labels = r.integers(0, 5, size=8)
        mb = T.sample(g, seeds, [3, 3], it)
        ra = O.iteration(mb.copy(), it, ca, lambda ids: X[ids], weights, None, 0.5, dims, labels=labels)
        rb = O.iteration(mb.copy(), it, cb, lambda ids: X[ids], weights, ra["backward"]["gnorm"], 0.5, dims)
        assert ra["stats"] == rb["stats"] and np.array_equal(ca[1].map, cb[1].map)
    assert ca[1].head > 0
