"""Pins of the oracle's mixed-precision setting (fp16 raw features, bf16 operands of every matrix product, bf16
embeddings between the layers, fp32 output of the last layer: the very large workload) and of the GCN backward pass.
No GPU.

What the pins compare the oracle with: a hand-worked example (tests/golden/mixed_precision_worked_example.txt);
identity-panel weights, under which a layer's output is one rounded operand, bit for bit; exact rational arithmetic
(`fractions`) for the means and the products; torch's CPU bfloat16 conversion as the rounding routine (the oracle has
its own); central finite differences for the GCN backward pass.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from fg_inputs.sampler import MiniBatch
from oracle import freshgnn_oracle as O
from tests import helpers as T


def bf16(x):
    """fp64 -> fp32 -> bfloat16 (nearest, ties to even) by torch's CPU conversion, returned as fp32 values."""
    t = torch.from_numpy(np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32)))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def is_bf16(x):
    return bool(np.all((np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) & 0xFFFF) == 0))


def exact_mean(rows):
    """Correctly rounded fp64 mean of a few fp16/bf16 rows, by rational arithmetic."""
    rows = np.asarray(rows, dtype=np.float64)
    return np.array([float(sum(Fraction(float(v)) for v in rows[:, k]) / len(rows)) for k in range(rows.shape[1])])


def exact_dot_f32(x, w, b):
    """fp32 value nearest to sum_k x_k w_k + b, by rational arithmetic."""
    z = sum(Fraction(float(a)) * Fraction(float(c)) for a, c in zip(x, w)) + Fraction(float(b))
    return np.float32(float(z))     # Fraction -> fp64 is correctly rounded; the second rounding can differ from a
                                    # direct one only at fp64-level near-ties, which these cases do not contain


# ---------------------------------------------------------------- hand-worked example

def load_worked_example():
    rows = {}
    for line in open(os.path.join(T.GOLDEN, "mixed_precision_worked_example.txt")):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            rows.setdefault(key, []).append(vals)
    f = lambda vals: [float(Fraction(v)) for v in vals]
    ex = dict(X=np.array([f(v[1:]) for v in rows["x"]]).astype(np.float16),
              W1=np.array([f(v) for v in rows["W1"]], dtype=np.float32), b1=np.array(f(rows["b1"][0]), dtype=np.float32),
              W2=np.array([f(v) for v in rows["W2"]], dtype=np.float32), b2=np.array(f(rows["b2"][0]), dtype=np.float32),
              AGG1=np.array([f(v[1:]) for v in rows["AGG1"]]), H1=np.array([f(v[1:]) for v in rows["H1"]]),
              H2=np.array([f(v[1:]) for v in rows["H2"]]))
    assert np.array_equal(ex["X"].astype(np.float64), np.array([f(v[1:]) for v in rows["x"]])), "the features are fp16 numbers"
    return ex


def worked_minibatch():
    ids = [np.array([0, 1, 2], np.int32), np.array([0, 1], np.int32), np.array([0], np.int32)]
    start = [None, np.array([0, 2], np.int32), np.array([0], np.int32)]
    end = [None, np.array([2, 3], np.int32), np.array([1], np.int32)]
    col = [None, np.array([1, 2, 2], np.int32), np.array([1], np.int32)]
    return MiniBatch(2, ids, start, end, col)


def test_worked_example_of_the_rounding_points():
    ex = load_worked_example()
    mb = worked_minibatch()
    O.check_minibatch(mb)
    weights = {1: (ex["W1"], ex["b1"]), 2: (ex["W2"], ex["b2"])}
    rec = O.iteration(mb, 0, {}, lambda ids: ex["X"][ids], weights, {}, 0.5, [2, 2, 1], feat_dtype="f16", compute_dtype="bf16")
    assert rec["H"][0].dtype == np.float16 and np.array_equal(rec["H"][0], ex["X"])
    assert np.array_equal(rec["AGG"][1], ex["AGG1"])                 # the mean is rounded to bf16 (one of them at a tie)
    assert np.array_equal(rec["H"][1], ex["H1"]) and is_bf16(rec["H"][1])
    assert rec["H"][2].dtype == np.float32 and not is_bf16(rec["H"][2])     # the last layer is not rounded to bf16
    assert np.array_equal(rec["H"][2], ex["H2"].astype(np.float32)) and float(rec["H"][2][0, 0]) == float(ex["H2"][0, 0])


# ---------------------------------------------------------------- identity panels: a layer's output is one rounded operand

def mixed_case(seed, L=2, n=80, d=8):
    g = T.random_explicit_graph(n, 6, seed, allow_isolated=True)
    r = np.random.default_rng(seed)
    X = (r.standard_normal((n, d)) * 1.7).astype(np.float16)
    seeds = r.permutation(n)[:12]
    mb = T.sample(g, seeds, [4] * L, 0)
    return g, X, mb, r


@pytest.mark.parametrize("seed", [0, 1])
def test_identity_panels_show_each_rounded_operand_bit_for_bit(seed):
    d = 8
    g, X, mb, r = mixed_case(seed, d=d)
    I, Z, zero = np.eye(d, dtype=np.float32), np.zeros((d, d), np.float32), np.zeros(d, np.float32)
    own_panel, neigh_panel = np.vstack([I, Z]), np.vstack([Z, I])
    run = lambda W1, W2: O.iteration(mb.copy(), 0, {}, lambda ids: X[ids], {1: (W1, zero), 2: (W2, zero)}, {}, 0.5, [d, d, d],
                                     feat_dtype="f16", compute_dtype="bf16")
    n1, n2 = len(mb.ids[1]), len(mb.ids[2])
    x64 = X.astype(np.float64)
    assert not is_bf16(X[mb.ids[1]].astype(np.float32)), "the case was meant to have fp16 values that are not bf16 numbers"

    # W1 = [I; 0]: H(1) = ReLU(bf16(own fp16 row))
    rec = run(own_panel, own_panel)
    want1 = np.maximum(bf16(x64[mb.ids[1]]), 0)
    assert rec["H"][1].dtype == np.float32 and np.array_equal(rec["H"][1], want1)
    # ... and the last layer with [I; 0] hands the seeds' rows through, as fp32
    assert rec["H"][2].dtype == np.float32 and np.array_equal(rec["H"][2], want1[:n2])

    # W1 = [0; I]: H(1) = ReLU(bf16(mean of the sampled neighbours' fp16 rows)), the mean correctly rounded
    rec = run(neigh_panel, neigh_panel)
    mean1 = np.zeros((n1, d))
    for j in range(n1):
        nb = mb.col[1][mb.start[1][j]:mb.end[1][j]]
        if len(nb):
            mean1[j] = exact_mean(x64[mb.ids[0][nb]])
    assert np.array_equal(rec["AGG"][1], bf16(mean1))
    assert not np.array_equal(bf16(mean1), mean1.astype(np.float32)), "the case was meant to have means that bf16 changes"
    h1 = np.maximum(bf16(mean1), 0)
    assert np.array_equal(rec["H"][1], h1)
    # last layer with [0; I]: bf16(mean of the bf16 rows of H(1)), stored as fp32
    mean2 = np.zeros((n2, d))
    for j in range(n2):
        nb = mb.col[2][mb.start[2][j]:mb.end[2][j]]
        if len(nb):
            mean2[j] = exact_mean(h1[nb])
    assert np.array_equal(rec["AGG"][2], bf16(mean2))
    assert np.array_equal(rec["H"][2], bf16(mean2))
    assert not np.array_equal(bf16(mean2), mean2.astype(np.float32))


def test_products_take_bf16_operands_and_the_last_layer_keeps_fp32():
    """General weights: every output equals the exactly computed sum of bf16(x)·bf16(w) + b, rounded once: to bf16
    below the last layer, to fp32 at the last layer. W is passed with more bits than bf16 holds."""
    d = 8
    g, X, mb, r = mixed_case(5, d=d)
    dims = [d, 6, 5]
    weights = T.random_weights(dims, 3)          # fp32 values, not bf16 numbers
    assert not is_bf16(weights[1][0])
    rec = O.iteration(mb.copy(), 0, {}, lambda ids: X[ids], weights, {}, 0.5, dims, feat_dtype="f16", compute_dtype="bf16")
    H_prev = X[mb.ids[0]].astype(np.float64)
    for l in (1, 2):
        W, b = weights[l]
        Wb = bf16(W).astype(np.float64)
        n = len(mb.ids[l])
        out = np.zeros((n, dims[l]), np.float32)
        for j in range(n):
            nb = mb.col[l][mb.start[l][j]:mb.end[l][j]]
            mean = exact_mean(H_prev[nb]) if len(nb) else np.zeros(dims[l - 1])
            xin = np.concatenate([bf16(H_prev[j]), bf16(mean)]).astype(np.float64)
            for c in range(dims[l]):
                z = exact_dot_f32(xin, Wb[:, c], b[c])
                out[j, c] = max(z, np.float32(0)) if l < 2 else z
        if l < 2:
            out = bf16(out)
            assert is_bf16(rec["H"][l]) and np.array_equal(rec["H"][l], out)
        else:
            assert rec["H"][l].dtype == np.float32 and not is_bf16(rec["H"][l])
            assert np.array_equal(rec["H"][l], out)
        H_prev = out.astype(np.float64)


def test_cached_rows_are_bf16_and_fetched_bit_for_bit():
    d = 8
    g = T.random_explicit_graph(60, 5, 2)
    r = np.random.default_rng(2)
    X = r.standard_normal((60, d)).astype(np.float16)
    dims = [d, 6, 6, 4]
    weights = T.random_weights(dims, 1)
    caches = {l: O.HistoricalCache(60, 40, dims[l], 4, "bf16") for l in (1, 2)}
    hits = 0
    for it in range(6):
        mb = T.sample(g, r.permutation(60)[:10], [3, 3, 3], it)
        gn = {l: np.exp(r.standard_normal(len(mb.ids[l]))).astype(np.float32) for l in (1, 2)}
        before = {l: caches[l].table.copy() for l in (1, 2)}
        rec = O.iteration(mb, it, caches, lambda ids: X[ids], weights, gn, 0.8, dims, feat_dtype="f16", compute_dtype="bf16")
        for l in (1, 2):
            for p, s in zip(rec["look"][l]["hit_pos"], rec["look"][l]["hit_slot"]):
                assert np.array_equal(rec["H"][l][p], before[l][s])
                hits += 1
            assert is_bf16(caches[l].table)
    assert hits > 0


# ---------------------------------------------------------------- backward pass in the mixed-precision setting

def backward_case(seed=3):
    d = 8
    g, X, mb, r = mixed_case(seed, d=d)
    dims = [d, 6, 5]
    weights = {l: (bf16(W), b) for l, (W, b) in T.random_weights(dims, seed).items()}
    labels = r.integers(0, dims[2], size=len(mb.ids[2]))
    return X, mb, dims, weights, labels


def test_backward_rounds_the_output_gradient_before_both_products():
    """With W_2 = [I; 0] the gradient handed to a seed's own previous embedding is bf16(dz) itself; with [0; I] every
    sampled neighbour receives bf16(dz)/deg. The weight gradient is [bf16(own) ‖ bf16(mean)]^T bf16(dz), the bias
    gradient sums the unrounded dz."""
    X, mb, dims, weights, labels = backward_case()
    d1, d2 = dims[1], dims[2]
    assert d1 >= d2
    n2 = len(mb.ids[2])
    for panel in ("own", "neigh"):
        W2 = np.zeros((2 * d1, d2), np.float32)
        W2[(0 if panel == "own" else d1) + np.arange(d2), np.arange(d2)] = 1.0
        ws = {1: weights[1], 2: (W2, weights[2][1])}
        rec = O.iteration(mb.copy(), 0, {}, lambda ids: X[ids], ws, None, 0.5, dims, feat_dtype="f16", compute_dtype="bf16", labels=labels)
        bw = rec["backward"]
        # dL/dH(2) by the definition of the loss: (softmax - onehot) / n on the fp32 outputs
        h = rec["H"][2].astype(np.float64)
        p = np.exp(h - h.max(1, keepdims=True))
        p /= p.sum(1, keepdims=True)
        p[np.arange(n2), labels] -= 1
        dz = p / n2
        np.testing.assert_allclose(bw["dH"][2], dz, rtol=1e-12, atol=0)
        dzb = bf16(dz).astype(np.float64)
        assert not np.array_equal(dzb, dz.astype(np.float32)), "the case was meant to have gradients that bf16 changes"
        want = np.zeros((len(mb.ids[1]), d1))
        for j in range(n2):
            if panel == "own":
                want[j, :d2] += dzb[j]
            else:
                nb = mb.col[2][mb.start[2][j]:mb.end[2][j]]
                for c in nb:
                    want[c, :d2] += dzb[j] / len(nb)
        np.testing.assert_allclose(bw["dH"][1], want, rtol=1e-14, atol=0)
        assert np.array_equal(bw["gnorm"][1], np.sqrt((want * want).sum(1)).astype(np.float32))
        x = np.concatenate([bf16(rec["H"][1][:n2]), rec["AGG"][2]], axis=1).astype(np.float64)
        np.testing.assert_allclose(bw["dW"][2], x.T @ dzb, rtol=1e-12, atol=1e-300)
        np.testing.assert_allclose(bw["db"][2], dz.astype(np.float32).astype(np.float64).sum(0), rtol=1e-12)   # dH is carried as fp32
        assert not np.allclose(bw["db"][2], dzb.sum(0), rtol=1e-6, atol=0)


def test_backward_of_a_lower_layer_masks_then_rounds_and_uses_rounded_weights():
    X, mb, dims, weights, labels = backward_case(4)
    ws = {1: weights[1], 2: (weights[2][0] * np.float32(1 + 2.0 ** -10), weights[2][1])}   # W_2 with bits beyond bf16
    ws3 = dict(ws)
    rec = O.iteration(mb.copy(), 0, {}, lambda ids: X[ids], ws3, None, 0.5, dims, feat_dtype="f16", compute_dtype="bf16", labels=labels)
    bw = rec["backward"]
    n2 = len(mb.ids[2])
    W2b = bf16(ws[2][0]).astype(np.float64)
    dzb = bf16(bw["dH"][2]).astype(np.float64)
    dx = dzb @ W2b.T
    want = np.zeros((len(mb.ids[1]), dims[1]))
    for j in range(n2):
        want[j] += dx[j, :dims[1]]
        nb = mb.col[2][mb.start[2][j]:mb.end[2][j]]
        for c in nb:
            want[c] += dx[j, dims[1]:] / len(nb)
    np.testing.assert_allclose(bw["dH"][1], want, rtol=1e-12, atol=1e-300)
    # layer 1: dz = bf16(fp32(dH(1)) masked by H(1) > 0); dW_1 = [bf16(x_own) ‖ bf16(mean)]^T dz
    rows = rec["look"][1]["normal_pos"]
    mask = rec["H"][1][rows] > 0
    assert mask.any() and not mask.all()
    dz1 = want.astype(np.float32).astype(np.float64)[rows] * mask
    x = np.concatenate([bf16(X[mb.ids[0][rows]].astype(np.float64)), rec["AGG"][1]], axis=1).astype(np.float64)
    np.testing.assert_allclose(bw["dW"][1], x.T @ bf16(dz1).astype(np.float64), rtol=1e-11, atol=1e-300)
    np.testing.assert_allclose(bw["db"][1], dz1.sum(0), rtol=1e-12, atol=1e-300)


def test_mixed_precision_backward_is_the_plain_one_when_nothing_needs_rounding():
    """Operands that are bf16 numbers already (small integers): the two settings must give identical gradients."""
    g = T.random_explicit_graph(40, 4, 7)
    r = np.random.default_rng(7)
    d = 4
    X = r.integers(-2, 3, size=(40, d)).astype(np.float16)
    mb = T.sample(g, r.permutation(40)[:6], [2, 2], 0)
    weights = {1: (r.integers(-1, 2, size=(2 * d, d)).astype(np.float32), np.zeros(d, np.float32)),
               2: (r.integers(-1, 2, size=(2 * d, 3)).astype(np.float32), np.zeros(3, np.float32))}
    # degrees 1 and 2 only keep the means at multiples of 1/2: bf16 numbers
    labels = r.integers(0, 3, size=6)
    a = O.iteration(mb.copy(), 0, {}, lambda ids: X[ids], weights, None, 0.5, [d, d, 3], feat_dtype="f16", compute_dtype="bf16", labels=labels)
    b = O.iteration(mb.copy(), 0, {}, lambda ids: X[ids].astype(np.float32), weights, None, 0.5, [d, d, 3], labels=labels)
    if not (is_bf16(a["H"][1]) and np.array_equal(a["H"][1], b["H"][1])):
        pytest.skip("this draw produced a hidden value that bf16 changes")
    assert np.array_equal(a["H"][2], b["H"][2])
    # dH is carried as fp32 in the bf16 setting: each of the 6 summed rows is off by at most half an fp32 ulp of an entry <= 1/6,
    # and the column sums cancel, so the bar is absolute
    np.testing.assert_allclose(a["backward"]["db"][2], b["backward"]["db"][2], rtol=0, atol=6 * 2.0 ** -25 / 6)
    np.testing.assert_allclose(a["backward"]["db"][1], b["backward"]["db"][1], rtol=1e-2)   # dz of layer 1 differs by the bf16 rounding only


# ---------------------------------------------------------------- GCN backward pass against finite differences

def gcn_forward_from(mb, rec, weights, l0, H_l0, W_override=None):
    L = mb.num_layers
    H = np.asarray(H_l0, dtype=np.float64)
    for l in range(l0 + 1, L + 1):
        rows = rec["look"][l]["normal_pos"]
        W, b = (W_override or weights)[l]
        out = np.asarray(rec["H"][l], dtype=np.float64).copy()
        out[rows] = O.linear_gcn(O.aggregate_gcn(mb.start[l], mb.end[l], mb.col[l], rows, H), W, b, relu=(l < L))
        H = out
    return H


def gcn_cached_run(seed):
    g = T.random_explicit_graph(100, 5, seed, allow_isolated=True)
    dims = [6, 7, 7, 5]            # a square weight matrix among them: W and its transpose must not be confused
    r = np.random.default_rng(seed)
    X = r.standard_normal((100, 6)).astype(np.float32)
    weights = {l: ((r.standard_normal((dims[l - 1], dims[l])) / np.sqrt(dims[l - 1])).astype(np.float32),
                   (0.1 * r.standard_normal(dims[l])).astype(np.float32)) for l in (1, 2, 3)}
    caches = {l: O.HistoricalCache(100, 60, dims[l], 3) for l in (1, 2)}
    for it in range(5):
        seeds = r.permutation(100)[:10]
        labels = r.integers(0, 5, size=10)
        mb = T.sample(g, seeds, [3, 3, 3], it)
        rec = O.iteration(mb, it, caches, lambda ids: X[ids], weights, None, 0.7, dims, labels=labels, model="gcn")
    return mb, rec, weights, labels, dims


@pytest.mark.parametrize("seed", [0, 1])
def test_gcn_gradients_against_finite_differences(seed):
    mb, rec, weights, labels, dims = gcn_cached_run(seed)
    bw = rec["backward"]
    L = 3
    assert sum(len(rec["look"][l]["hit_pos"]) for l in (1, 2)) > 0
    loss = lambda l, H, ws=None: O.softmax_xent(gcn_forward_from(mb, rec, weights, l, H, ws), labels)
    eps = 1e-5
    r = np.random.default_rng(seed)
    for l in (1, 2, 3):
        base = np.asarray(rec["H"][l], dtype=np.float64)
        assert abs(loss(l, base) - O.softmax_xent(rec["H"][L], labels)) < 1e-5
        for j in r.permutation(len(base))[:10]:
            for c in r.permutation(dims[l])[:2]:
                hp, hm = base.copy(), base.copy()
                hp[j, c] += eps
                hm[j, c] -= eps
                num = (loss(l, hp) - loss(l, hm)) / (2 * eps)
                assert abs(num - bw["dH"][l][j, c]) < 1e-7 + 1e-4 * abs(num), (l, j, c)
        live = rec["live"][l] if rec["live"][l] is not None else np.ones(len(base), bool)
        assert not bw["dH"][l][~live].any()
        W, b = weights[l]
        prev = np.asarray(rec["H"][l - 1], dtype=np.float64)
        for _ in range(5):
            a, c = int(r.integers(0, W.shape[0])), int(r.integers(0, W.shape[1]))
            out = []
            for sgn in (1, -1):
                W2 = W.astype(np.float64).copy()
                W2[a, c] += sgn * eps
                ws = dict(weights)
                ws[l] = (W2, b)
                out.append(loss(l - 1, prev, ws))
            num = (out[0] - out[1]) / (2 * eps)
            assert abs(num - bw["dW"][l][a, c]) < 1e-7 + 1e-4 * abs(num)
        c = int(r.integers(0, len(b)))
        out = []
        for sgn in (1, -1):
            b2 = b.astype(np.float64).copy()
            b2[c] += sgn * eps
            ws = dict(weights)
            ws[l] = (W, b2)
            out.append(loss(l - 1, prev, ws))
        assert abs((out[0] - out[1]) / (2 * eps) - bw["db"][l][c]) < 1e-7
    for l in (1, 2):
        assert np.allclose(bw["gnorm"][l], np.linalg.norm(bw["dH"][l], axis=1), rtol=1e-6)
