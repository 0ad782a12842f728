"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test compares the oracle with something that is not the oracle: a dense whole-graph
recursion of Eq. 1, closed forms, a depth-first needed-set, an eager dictionary model of the
cache, and hand-worked traces stored under tests/golden.
"""
import numpy as np
import pytest

from oracle import freshgnn_oracle as O
from tests import helpers as T


def run_iteration(g, seeds, fanouts, it, caches, X, weights, dims, p_grad=0.5, gn_seed=11, update=True, sample_seed=7):
    mb = T.sample(g, seeds, fanouts, it, seed=sample_seed)
    O.check_minibatch(mb)
    r = np.random.default_rng(gn_seed * 1000 + it)
    gn = {l: np.exp(r.standard_normal(len(mb.ids[l]))).astype(np.float32) for l in range(1, len(fanouts))}
    rec = O.iteration(mb, it, caches, lambda ids: X[ids], weights, gn, p_grad, dims, update=update)
    return mb, rec


def dense_forward(g, X, weights, L):
    """H^(l) = act([H^(l-1) ‖ D^-1 A H^(l-1)] W_l + b_l) for every node of the graph (Eq. 1, mean aggregator)."""
    A = T.dense_adjacency(g)
    deg = A.sum(axis=1, keepdims=True)
    P = np.divide(A, deg, out=np.zeros_like(A), where=deg > 0)
    H = X.astype(np.float64)
    for l in range(1, L + 1):
        W, b = weights[l]
        Z = np.concatenate([H, P @ H], axis=1) @ W.astype(np.float64) + b.astype(np.float64)
        H = np.maximum(Z, 0) if l < L else Z
    return H


# ---------------------------------------------------------------- Eq. 1 against the dense recursion

@pytest.mark.parametrize("L,seed", [(1, 0), (2, 1), (3, 2)])
def test_full_neighbourhood_equals_dense_recursion(L, seed):
    g = T.random_explicit_graph(60, 5, seed)
    dims = [6] + [5, 7, 4][:L]
    X = np.random.default_rng(seed).standard_normal((60, dims[0])).astype(np.float32)
    weights = T.random_weights(dims, seed + 1)
    seeds = np.random.default_rng(seed + 2).permutation(60)[:9]
    mb, rec = run_iteration(g, seeds, [5] * L, 0, {}, X, weights, dims)
    want = dense_forward(g, X, weights, L)[seeds]
    got = rec["H"][L]
    assert got.dtype == np.float32
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6 * np.abs(want).max())


def test_intermediate_layers_equal_dense_recursion():
    g = T.random_explicit_graph(40, 4, 5, allow_isolated=True)
    dims = [5, 6, 3]
    X = np.random.default_rng(3).standard_normal((40, 5)).astype(np.float32)
    weights = T.random_weights(dims, 4)
    mb, rec = run_iteration(g, np.arange(0, 40, 5), [4, 4], 0, {}, X, weights, dims)
    H1 = dense_forward(g, X, {1: weights[1], 2: weights[2]}, 2)  # last layer
    A = T.dense_adjacency(g)
    deg = A.sum(1, keepdims=True)
    P = np.divide(A, deg, out=np.zeros_like(A), where=deg > 0)
    W, b = weights[1]
    layer1 = np.maximum(np.concatenate([X.astype(np.float64), P @ X], 1) @ W + b, 0)
    live1 = rec["live"][1]
    np.testing.assert_allclose(rec["H"][1][live1], layer1[mb.ids[1][live1]], atol=3e-6)
    np.testing.assert_allclose(rec["H"][2], H1[mb.ids[2]], atol=3e-6)
    # isolated rows: the neighbour mean is the zero vector
    iso = [k for k, r in enumerate(rec["look"][1]["normal_pos"]) if mb.end[1][r] == mb.start[1][r]]
    assert all(np.all(rec["AGG"][1][k] == 0) for k in iso)


# ---------------------------------------------------------------- closed forms of the aggregator and the linear

def test_mean_closed_forms():
    start = np.array([0, 3, 3, 5]); end = np.array([3, 3, 5, 9]); col = np.array([0, 2, 4, 1, 1, 0, 1, 2, 3])
    const = np.full((5, 3), 2.5, dtype=np.float32)
    out = O.aggregate(start, end, col, [0, 1, 2, 3], const)
    assert np.array_equal(out[[0, 2, 3]], np.full((3, 3), 2.5)) and np.all(out[1] == 0)
    onehot = np.eye(5, dtype=np.float32)
    out = O.aggregate(start, end, col, [0, 2, 3], onehot)
    np.testing.assert_allclose(out[0], [1 / 3, 0, 1 / 3, 0, 1 / 3])
    np.testing.assert_allclose(out[1], [0, 1, 0, 0, 0])          # neighbour 1 twice: mean of two equal rows
    np.testing.assert_allclose(out[2], [.25, .25, .25, .25, 0])
    # only the listed rows are produced, in list order
    out = O.aggregate(start, end, col, [3, 0], onehot)
    np.testing.assert_allclose(out[1], [1 / 3, 0, 1 / 3, 0, 1 / 3])


def test_linear_panels_and_activation():
    r = np.random.default_rng(0)
    hs = r.standard_normal((7, 4)); ag = r.standard_normal((7, 4))
    I, Z = np.eye(4), np.zeros((4, 4))
    zero = np.zeros(4)
    assert np.array_equal(O.linear(hs, ag, np.vstack([I, Z]), zero, relu=False), hs)      # own panel first
    assert np.array_equal(O.linear(hs, ag, np.vstack([Z, I]), zero, relu=False), ag)      # neighbour panel second
    assert np.array_equal(O.linear(hs, ag, np.vstack([I, Z]), zero, relu=True), np.maximum(hs, 0))
    b = np.array([1., -2., 3., 0.5])
    assert np.array_equal(O.linear(hs, ag, np.vstack([Z, Z]), b, relu=False), np.tile(b, (7, 1)))
    W = r.standard_normal((8, 3))
    want = np.array([[sum(hs[i, k] * W[k, j] for k in range(4)) + sum(ag[i, k] * W[4 + k, j] for k in range(4))
                      for j in range(3)] for i in range(7)])
    np.testing.assert_allclose(O.linear(hs, ag, W, np.zeros(3), relu=False), want, atol=1e-12)


def test_bf16_rounding_points():
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: ties go to even (1.0); slightly above goes up
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -16, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8, 3.0e38])
    got = O.round_bf16(x)
    assert got.tolist()[:4] == [1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -1.0]
    assert np.all((got.view(np.uint32) & 0xFFFF) == 0)


# ---------------------------------------------------------------- pruning against a depth-first needed-set

def needed_sets(mb, cached):
    """Brute force: walk down from the seeds through the sampled edges, stopping below cached nodes."""
    L = mb.num_layers
    need = [set() for _ in range(L + 1)]
    hit = [set() for _ in range(L + 1)]

    def visit(l, j):
        if j in need[l]:
            return
        need[l].add(j)
        v = int(mb.ids[l][j])
        if 1 <= l <= L - 1 and v in cached.get(l, ()):
            hit[l].add(j)
            return
        if l >= 1:
            visit(l - 1, j)
            for e in range(mb.start[l][j], mb.end[l][j]):
                visit(l - 1, int(mb.col[l][e]))

    for j in range(len(mb.ids[L])):
        visit(L, j)
    return need, hit


@pytest.mark.parametrize("seed", range(4))
def test_prune_matches_depth_first_needed_set(seed):
    g = T.random_explicit_graph(300, 8, seed)
    L = 3
    dims = [4, 4, 4, 4]
    X = np.random.default_rng(seed).standard_normal((300, 4)).astype(np.float32)
    weights = T.random_weights(dims, seed)
    caches = {l: O.HistoricalCache(300, 200, 4, 5) for l in (1, 2)}
    seeds0 = np.random.default_rng(seed).permutation(300)[:40]
    run_iteration(g, seeds0, [3, 3, 3], 0, caches, X, weights, dims, p_grad=0.7)   # fills the caches
    cached = {l: set(caches[l].valid_entries(1)) for l in (1, 2)}
    assert all(len(cached[l]) > 5 for l in cached)
    seeds1 = np.random.default_rng(seed + 100).permutation(300)[:40]
    pristine = T.sample(g, seeds1, [3, 3, 3], 1)
    need, hit = needed_sets(pristine, cached)
    mb, rec = run_iteration(g, seeds1, [3, 3, 3], 1, caches, X, weights, dims, update=False)
    for l in range(L + 1):
        assert set(np.flatnonzero(rec["live"][l])) == need[l]
        assert set(rec["look"][l]["hit_pos"].tolist()) == hit[l]
        assert set(rec["look"][l]["normal_pos"].tolist()) == need[l] - hit[l]
        assert list(rec["look"][l]["normal_pos"]) == sorted(rec["look"][l]["normal_pos"])
    assert sum(len(h) for h in hit) > 0
    # two-row-array pruning: end == start exactly on rows that are not normal; col and start untouched
    for l in range(1, L + 1):
        normal = np.zeros(len(mb.ids[l]), bool); normal[rec["look"][l]["normal_pos"]] = True
        assert np.array_equal(mb.end[l][normal], pristine.end[l][normal])
        assert np.array_equal(mb.end[l][~normal], pristine.start[l][~normal])
        assert np.array_equal(mb.col[l], pristine.col[l]) and np.array_equal(mb.start[l], pristine.start[l])
    # pruning can only shrink the set of raw features loaded
    _, rec0 = run_iteration(g, seeds1, [3, 3, 3], 1, {}, X, weights, dims, update=False)
    assert len(rec["look"][0]["normal_pos"]) < len(rec0["look"][0]["normal_pos"])


# ---------------------------------------------------------------- exact-history invariant and degenerate settings

def _outputs_over_iterations(caches, p_grad, iters=8, L=3):
    g = T.random_explicit_graph(120, 4, 9, allow_isolated=False)
    dims = [5, 6, 6, 3][:L + 1]
    X = np.random.default_rng(1).standard_normal((120, 5)).astype(np.float32)
    weights = T.random_weights(dims, 2)
    outs, hits, nin = [], 0, []
    for it in range(iters):
        seeds = np.random.default_rng(50 + it).permutation(120)[:30]
        mb, rec = run_iteration(g, seeds, [4] * L, it, caches, X, weights, dims, p_grad=p_grad)
        outs.append(rec["H"][L].copy())
        hits += sum(len(rec["look"][l]["hit_pos"]) for l in range(1, L))
        nin.append(len(rec["look"][0]["normal_pos"]))
    return outs, hits, nin


def test_exact_history_invariant():
    """With fixed weights and full neighbourhoods a cached embedding equals the recomputed one,
    so any cache setting must reproduce the cache-free outputs (Eq. 2 becomes an equality)."""
    base, h0, n0 = _outputs_over_iterations({}, 0.5)
    assert h0 == 0
    for p_grad, t_stale, cap in [(0.5, 3, 64), (1.0, 100, 120), (0.8, 2, 7), (0.3, 1, 1)]:
        caches = {l: O.HistoricalCache(120, cap, 6, t_stale) for l in (1, 2)}
        outs, hits, nin = _outputs_over_iterations(caches, p_grad)
        assert hits > 0
        assert all(a <= b for a, b in zip(nin, n0)) and (cap < 60 or sum(nin) < sum(n0))
        for a, b in zip(outs, base):
            np.testing.assert_allclose(a, b, atol=2e-6)


@pytest.mark.parametrize("p_grad,t_stale", [(0.0, 5), (0.7, 0)])
def test_degenerate_settings_reduce_to_neighbour_sampling(p_grad, t_stale):
    """p_grad = 0 or t_stale = 0 is plain neighbour sampling (Section 4.1.3): no hit ever, identical outputs."""
    base, _, n0 = _outputs_over_iterations({}, 0.5)
    caches = {l: O.HistoricalCache(120, 50, 6, t_stale) for l in (1, 2)}
    outs, hits, nin = _outputs_over_iterations(caches, p_grad)
    assert hits == 0 and nin == n0
    for a, b in zip(outs, base):
        assert np.array_equal(a, b)


def test_admit_everything_keeps_everything_computed():
    """p_grad = 1 with an unbounded staleness and room for all nodes keeps every computed embedding (Section 4.1.3)."""
    g = T.random_explicit_graph(150, 4, 3)
    dims = [4, 5, 5, 2]
    X = np.random.default_rng(1).standard_normal((150, 4)).astype(np.float32)
    weights = T.random_weights(dims, 2)
    caches = {l: O.HistoricalCache(150, 150, 5, 10 ** 6) for l in (1, 2)}
    seen = {1: {}, 2: {}}
    for it in range(10):
        seeds = np.random.default_rng(it).permutation(150)[:20]
        mb, rec = run_iteration(g, seeds, [2, 2, 2], it, caches, X, weights, dims, p_grad=1.0)
        for l in (1, 2):
            for j in rec["look"][l]["normal_pos"]:
                seen[l][int(mb.ids[l][j])] = rec["H"][l][j].copy()
            valid = caches[l].valid_entries(it + 1)
            assert set(valid) == set(seen[l])
            for v, (s, _) in valid.items():
                assert np.array_equal(caches[l].table[s], seen[l][v])


# ---------------------------------------------------------------- threshold

def test_threshold_is_rank_statistic_and_order_free():
    r = np.random.default_rng(0)
    g = np.exp(r.standard_normal(37)).astype(np.float32)
    for p in [0.0, 0.1, 0.3, 0.5, 0.9, 0.999, 1.0]:
        tau, k = O.admission_threshold(g, p)
        assert k == int(np.floor(np.float64(np.float32(p)) * 37))
        if k == 0:
            assert tau == -np.inf and not np.any(g < tau)
        elif k >= 37:
            assert tau == np.inf and np.all(g < tau)
        else:
            assert (g < tau).sum() == k        # distinct values: exactly the k smallest are below tau
            assert tau == sorted(g.tolist())[k]
        assert O.admission_threshold(r.permutation(g), p)[0] == tau
    # ties at the threshold are not admitted
    tied = np.array([1, 2, 2, 2, 3], dtype=np.float32)
    tau, k = O.admission_threshold(tied, 0.5)     # k = 2 -> tau = 2
    assert (k, tau) == (2, 2.0) and (tied < tau).sum() == 1
    assert O.admission_threshold(np.array([], dtype=np.float32), 0.5)[0] == -np.inf


# ---------------------------------------------------------------- hand-worked traces

def _drive_trace(name):
    params, steps = T.parse_trace(name)
    N = 32
    cache = O.HistoricalCache(N, params["capacity"], 2, params["t_stale"])
    for st in steps:
        i = st["iter"]
        ids = np.array([v for v, _ in st["live"]], dtype=np.int32)
        gn = np.array([x for _, x in st["live"]], dtype=np.float32)
        look = O.lookup_prune(cache, i, ids, None, None, None, None, 0)
        assert sorted(ids[look["hit_pos"]].tolist()) == sorted(st["hits"]), f"hits at iteration {i}"
        h = np.stack([np.full(2, 100.0 * i + v, dtype=np.float32) for v in ids])
        for p, s in zip(look["hit_pos"], look["hit_slot"]):
            h[p] = cache.table[s]
        O.cache_update(cache, i, ids, None, look["hit"], gn, params["p_grad"], h)
        valid = {v: stamp for v, (s, stamp) in cache.valid_entries(i + 1).items()}
        assert valid == st["valid_after"], f"valid set after iteration {i}"
        for v, (s, stamp) in cache.valid_entries(i + 1).items():
            assert np.all(cache.table[s] == 100.0 * stamp + v)     # the row stored is the one computed at admission
        if "slots" in st:
            assert cache.slot_node.tolist() == st["slots"]
        if "head" in st:
            assert cache.head == st["head"]


def test_trace_gradient_and_staleness():
    _drive_trace("cache_trace_gradient_staleness.txt")


def test_trace_ring():
    _drive_trace("cache_trace_ring.txt")


def test_staleness_boundary():
    """Admitted by the update of iteration a: usable at a+1 .. a+t_stale, gone at a+t_stale+1 (Section 4.1.2)."""
    for t_stale in (1, 4):
        c = O.HistoricalCache(10, 4, 1, t_stale)
        O.cache_update(c, 7, np.array([3]), None, np.array([False]), np.array([1.0], np.float32), 1.0, np.ones((1, 1), np.float32))
        assert c.slot_of(3, 7) == -1
        for i in range(8, 8 + t_stale):
            assert c.slot_of(3, i) == 0
        assert c.slot_of(3, 8 + t_stale) == -1


# ---------------------------------------------------------------- eager dictionary model of the cache

class DictModel:
    """Independent model: a dictionary of live entries with eager removal (no back-pointers)."""

    def __init__(self, capacity, t_stale):
        self.cap, self.t = capacity, t_stale
        self.where = {}                   # node -> slot
        self.ring = [None] * capacity     # slot -> (node, stamp, row)
        self.head = 0

    def hit(self, v, i):
        if v not in self.where:
            return False
        return 1 <= i - self.ring[self.where[v]][1] <= self.t

    def update(self, i, ids, live, gn, p, rows):
        pop = [j for j in range(len(ids)) if live[j]]
        hits = {j for j in pop if self.hit(int(ids[j]), i)}
        k = int(np.floor(np.float64(np.float32(p)) * len(pop)))
        srt = sorted(float(gn[j]) for j in pop)
        low = (lambda x: False) if k <= 0 else (lambda x: True) if k >= len(pop) else (lambda x: x < srt[k])
        for j in hits:
            if not low(float(gn[j])):
                del self.where[int(ids[j])]
        adm = [j for j in pop if j not in hits and low(float(gn[j]))][: self.cap]
        for r, j in enumerate(adm):
            s = (self.head + r) % self.cap
            if self.ring[s] is not None and self.where.get(self.ring[s][0]) == s:
                del self.where[self.ring[s][0]]
            self.ring[s] = (int(ids[j]), i, rows[j].copy())
            self.where[int(ids[j])] = s
        self.head = (self.head + len(adm)) % self.cap


@pytest.mark.parametrize("cap,t_stale,p", [(5, 2, 0.5), (16, 4, 0.9), (3, 1, 1.0), (40, 50, 0.3)])
def test_cache_matches_dictionary_model(cap, t_stale, p):
    r = np.random.default_rng(cap * 100 + t_stale)
    N = 30
    c = O.HistoricalCache(N, cap, 3, t_stale)
    m = DictModel(cap, t_stale)
    for i in range(60):
        n = int(r.integers(0, 12))
        ids = r.permutation(N)[:n].astype(np.int32)
        live = r.random(n) < 0.8
        gn = np.round(np.exp(r.standard_normal(n)), 1).astype(np.float32)     # rounded: ties occur
        rows = r.standard_normal((n, 3)).astype(np.float32)
        look = O.lookup_prune(c, i, ids, live, None, None, None, 0)
        assert [int(ids[j]) for j in look["hit_pos"]] == [int(ids[j]) for j in range(n) if live[j] and m.hit(int(ids[j]), i)]
        O.cache_update(c, i, ids, live, look["hit"], gn, p, rows)
        m.update(i, ids, live, gn, p, rows)
        valid = c.valid_entries(i + 1)
        assert set(valid) == {v for v in m.where if m.hit(v, i + 1)}
        assert len(valid) <= cap
        for v, (s, stamp) in valid.items():
            assert c.map[v] == s and c.slot_node[s] == v and 1 <= i + 1 - stamp <= t_stale
            assert np.array_equal(c.table[s], m.ring[m.where[v]][2])
        assert c.head == m.head


# ---------------------------------------------------------------- stabilization period (Section 4.1.4)

def test_stabilization_period_is_plain_sampling_then_a_cache_that_starts_empty():
    g = T.random_explicit_graph(150, 5, 8)
    dims = [6, 7, 7, 4]
    X = np.random.default_rng(1).standard_normal((150, 6)).astype(np.float32)
    weights = T.random_weights(dims, 2)
    period = 4

    def run(stabilization, p_grad_of):
        caches = {l: O.HistoricalCache(150, 80, dims[l], 3) for l in (1, 2)}
        out = []
        for it in range(10):
            seeds = np.random.default_rng(100 + it).permutation(150)[:10]
            mb = T.sample(g, seeds, [3, 3, 3], it)
            r = np.random.default_rng(500 + it)
            gn = {l: np.exp(r.standard_normal(len(mb.ids[l]))).astype(np.float32) for l in (1, 2)}
            rec = O.iteration(mb, it, caches, lambda ids: X[ids], weights, gn, p_grad_of(it), dims, stabilization=stabilization)
            out.append((rec, mb))
        return out, caches

    with_period, ca = run(period, lambda it: 0.6)
    plain, _ = run(0, lambda it: 0.0)                       # p_grad = 0: neighbour sampling without a cache (Section 4.1.3)
    gated, cb = run(0, lambda it: 0.0 if it < period else 0.6)   # the same policy said differently: nothing admitted before `period`
    for it in range(10):
        a, b, c = with_period[it][0], plain[it][0], gated[it][0]
        if it < period:                                     # regular mini-batch training
            for l in range(4):
                assert np.array_equal(a["H"][l], b["H"][l])
            assert all(len(a["look"][l]["hit_pos"]) == 0 for l in (1, 2))
            assert all(a["stats"][l]["admitted"] == 0 for l in (1, 2))
        for l in range(1, 4):                               # afterwards: a cache that started empty at `period`
            assert np.array_equal(a["look"][l]["hit_pos"], c["look"][l]["hit_pos"])
            assert np.array_equal(a["H"][l], c["H"][l])
    assert sum(len(with_period[it][0]["look"][1]["hit_pos"]) for it in range(period + 1, 10)) > 0
    assert all(np.array_equal(ca[l].map, cb[l].map) and ca[l].head == cb[l].head for l in (1, 2))
    assert min(int(s) for l in (1, 2) for s in ca[l].slot_stamp[ca[l].slot_node >= 0]) >= period


# ---------------------------------------------------------------- GCN layers

def test_gcn_full_neighbourhood_equals_dense_recursion_and_closed_forms():
    """H = act(D~^-1 (A + I) H W + b): row-normalised graph convolution with self loops, over the whole graph."""
    g = T.random_explicit_graph(50, 5, 6)
    dims = [6, 5, 7, 4]
    L = 3
    X = np.random.default_rng(0).standard_normal((50, 6)).astype(np.float32)
    r = np.random.default_rng(1)
    weights = {l: ((r.standard_normal((dims[l - 1], dims[l])) / np.sqrt(dims[l - 1])).astype(np.float32),
                   (0.1 * r.standard_normal(dims[l])).astype(np.float32)) for l in range(1, L + 1)}
    seeds = np.random.default_rng(2).permutation(50)[:9]
    mb = T.sample(g, seeds, [5] * L, 0)
    rec = O.iteration(mb, 0, {}, lambda ids: X[ids], weights, {}, 0.5, dims, model="gcn")
    A = T.dense_adjacency(g) + np.eye(50)
    P = A / A.sum(axis=1, keepdims=True)
    H = X.astype(np.float64)
    for l in range(1, L + 1):
        Z = P @ H @ weights[l][0].astype(np.float64) + weights[l][1].astype(np.float64)
        H = np.maximum(Z, 0) if l < L else Z
    np.testing.assert_allclose(rec["H"][L], H[seeds], rtol=0, atol=2e-6 * np.abs(H).max())
    # closed forms of the propagation: an isolated row keeps its own embedding; constant features stay constant
    start, end, col = np.array([0, 0, 2]), np.array([0, 2, 3]), np.array([0, 2, 1])
    h = np.array([[1.0, 2.0], [3.0, 5.0], [7.0, 11.0]])
    got = O.aggregate_gcn(start, end, col, [0, 1, 2], h)
    assert np.allclose(got, [[1, 2], [(3 + 1 + 7) / 3, (5 + 2 + 11) / 3], [(7 + 3) / 2, (11 + 5) / 2]])
    assert np.allclose(O.aggregate_gcn(start, end, col, [2, 0], np.full((3, 4), 2.5)), 2.5)
    assert np.allclose(O.linear_gcn(np.eye(3), np.arange(6.0).reshape(3, 2), [1.0, -10.0], relu=True), [[1, 0], [3, 0], [5, 0]])
