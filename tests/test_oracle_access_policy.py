"""Pins of the access-aware admission (the policy "for accuracy and performance" of Section 7.4; no GPU).

The paper names what the policy prefers (embeddings that save more memory access) but neither the estimate nor the
rule, so these pins fix the reading taken against things that are not the oracle's code: an instrumented recursive
evaluation that counts the rows it touches, closed forms on full trees, the row count of the loader, a hand-worked
example, the rank definition of "the B best" by brute force, and an eager dictionary model of the cache.
"""
import numpy as np
import pytest

from oracle import freshgnn_oracle as O
from tests import helpers as T
from tests.test_oracle_pins import DictModel


def estimates(mb, look, upto):
    below, out = None, {}
    for l in range(1, upto + 1):
        out[l] = below = O.access_estimate(mb.start[l], mb.end[l], mb.col[l], look[l]["hit"], below)
    return out


# ---------------------------------------------------------------- the estimate

def rows_touched(mb, look, l, j):
    """Evaluate h_j^(l) the slow way, with no reuse of shared neighbours, and count the rows it reads."""
    if l == 0:
        return 1                                   # a raw feature row
    if look[l]["hit"][j]:
        return 1                                   # a cached embedding
    n = rows_touched(mb, look, l - 1, j)           # its own previous embedding
    for c in range(int(mb.start[l][j]), int(mb.end[l][j])):
        n += rows_touched(mb, look, l - 1, int(mb.col[l][c]))
    return n


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_estimate_counts_the_rows_an_unshared_evaluation_reads(seed):
    r = np.random.default_rng(seed)
    N, L, fan = 60, 3, (3, 3, 2)
    g = T.random_explicit_graph(N, 5, seed)
    dims = [4, 4, 4, 4]
    X = r.standard_normal((N, 4)).astype(np.float32)
    weights = T.random_weights(dims, seed)
    caches = {l: O.HistoricalCache(N, 40, dims[l], 5) for l in (1, 2)}
    seen_hit = False
    for it in range(6):
        mb = T.sample(g, r.permutation(N)[:8], fan, it, seed=seed)
        gn = {l: np.exp(r.standard_normal(len(mb.ids[l]))).astype(np.float32) for l in (1, 2)}
        rec = O.iteration(mb, it, caches, lambda ids: X[ids], weights, gn, 0.7, dims, admit_budget={1: 1000, 2: 1000})
        look = rec["look"]
        for l in (1, 2):
            seen_hit |= bool(look[l]["hit"].any())
            for j in look[l]["normal_pos"].tolist() + look[l]["hit_pos"].tolist():
                assert rec["saving"][l][j] == min(rows_touched(mb, look, l, j), O.SAVING_MAX)
        # what the loader reads for layer 1 is the sum of the estimates of its computed rows
        normal = look[1]["normal_pos"]
        assert int(rec["saving"][1][normal].sum()) == len(normal) + int((mb.end[1] - mb.start[1])[normal].sum())
    assert seen_hit


def test_estimate_on_full_trees_is_a_product_and_saturates():
    """Every row with exactly f_l neighbours and no hit: (1 + f_1) ... (1 + f_l), whatever the columns are."""
    r = np.random.default_rng(5)
    n = [40, 20, 8, 3]                  # nodes of layers 0..3
    f = [None, 4, 6, 90]
    below = None
    for l in (1, 2, 3):
        start = np.arange(n[l]) * f[l]
        col = r.integers(0, n[l - 1], size=n[l] * f[l])
        a = O.access_estimate(start, start + f[l], col, np.zeros(n[l], dtype=bool), below)
        expect = np.prod([1 + f[k] for k in range(1, l + 1)])
        assert np.all(a == min(expect, O.SAVING_MAX))
        below = a
    assert O.SAVING_MAX == 2047 and (1 + 4) * (1 + 6) * (1 + 90) > O.SAVING_MAX


def test_estimate_hand_example():
    """Layer 1: rows 0..3 over sources 0..5; row 1 was pruned by a hit above it (no neighbours left), row 2 is a hit.
    Layer 2: rows 0..1 over layer 1; row 1 is a hit.
        a1 = [1 + 3, 1 + 0, 1 (hit), 1 + 2] = [4, 1, 1, 3]
        a2[0] = a1[0] + a1[1] + a1[2] + a1[3] = 9;  a2[1] = 1 (hit)"""
    s1, e1 = np.array([0, 3, 3, 5]), np.array([3, 3, 5, 7])
    c1 = np.array([4, 5, 1, 0, 4, 2, 5])
    a1 = O.access_estimate(s1, e1, c1, np.array([False, False, True, False]))
    assert a1.tolist() == [4, 1, 1, 3]
    s2, e2 = np.array([0, 3]), np.array([3, 3])
    a2 = O.access_estimate(s2, e2, np.array([1, 2, 3]), np.array([False, True]), a1)
    assert a2.tolist() == [9, 1]


# ---------------------------------------------------------------- the admission rule

def fresh(cap, N=64, d=2, t_stale=9):
    return O.HistoricalCache(N, cap, d, t_stale)


def admitted_nodes(cache, it):
    return {v: s for v, (s, stamp) in cache.valid_entries(it + 1).items() if stamp == it}


def test_admission_hand_example():
    """Six admissible nodes with estimates 3 5 5 1 5 2: a budget of 3 takes positions 1, 2, 4 (the three fives), a budget
    of 4 adds position 0; rows go into consecutive slots in position order; the others are counted as dropped."""
    ids = np.array([10, 11, 12, 13, 14, 15], dtype=np.int32)
    gn = np.full(6, 0.5, dtype=np.float32)
    rows = np.arange(12, dtype=np.float32).reshape(6, 2)
    hit = np.zeros(6, dtype=bool)
    saving = np.array([3, 5, 5, 1, 5, 2])
    for budget, expect in ((3, [11, 12, 14]), (4, [10, 11, 12, 14]), (6, [10, 11, 12, 13, 14, 15]), (0, [])):
        c = fresh(8)
        c.head = 6
        st = O.cache_update(c, 0, ids, None, hit, gn, 1.0, rows, saving=saving, budget=budget)
        adm = admitted_nodes(c, 0)
        assert sorted(adm) == expect and st["admitted"] == len(expect) and st["dropped_overflow"] == 6 - len(expect)
        assert [adm[v] for v in expect] == [(6 + r) % 8 for r in range(len(expect))]
        for v in expect:
            assert np.array_equal(c.table[adm[v]], rows[v - 10])
        assert c.head == (6 + len(expect)) % 8
    # ties beyond the budget: the lower positions win
    c = fresh(8)
    O.cache_update(c, 0, ids, None, hit, gn, 1.0, rows, saving=np.array([5, 5, 5, 5, 5, 5]), budget=2)
    assert sorted(admitted_nodes(c, 0)) == [10, 11]
    # the budget cannot exceed the ring
    c = fresh(4)
    st = O.cache_update(c, 0, ids, None, hit, gn, 1.0, rows, saving=saving, budget=100)
    assert sorted(admitted_nodes(c, 0)) == [10, 11, 12, 14] and st["dropped_overflow"] == 2
    # estimates above the saturation point are equal
    c = fresh(8)
    O.cache_update(c, 0, ids, None, hit, gn, 1.0, rows, saving=np.array([2047, 9000, 1, 5000, 2046, 3000]), budget=2)
    assert sorted(admitted_nodes(c, 0)) == [10, 11]


@pytest.mark.parametrize("seed", range(6))
def test_admission_is_the_rank_definition(seed):
    """j gets in iff fewer than B admissible nodes have a larger estimate or an equal one at a lower position; hits
    and the gradient rule are untouched by the budget."""
    r = np.random.default_rng(100 + seed)
    N, n = 200, 90
    cap = int(r.integers(20, 120))
    c = fresh(cap, N=N)
    plain = fresh(cap, N=N)
    for it in range(5):
        ids = r.permutation(N)[:n].astype(np.int32)
        live = r.random(n) < 0.85
        gn = np.round(np.exp(r.standard_normal(n)), 1).astype(np.float32)
        saving = r.integers(1, 12, size=n)
        rows = r.standard_normal((n, 2)).astype(np.float32)
        budget = int(r.integers(0, 60))
        look = O.lookup_prune(c, it, ids, live, None, None, None, 0)
        tau, _ = O.admission_threshold(gn[live], 0.8)
        cand = [j for j in range(n) if live[j] and not look["hit"][j] and gn[j] < tau]
        room = min(budget, cap)
        expect = [j for j in cand
                  if sum(1 for k in cand if saving[k] > saving[j] or (saving[k] == saving[j] and k < j)) < room]
        before = dict(c.valid_entries(it + 1))
        st = O.cache_update(c, it, ids, live, look["hit"], gn, 0.8, rows, saving=saving, budget=budget)
        adm = admitted_nodes(c, it)
        assert sorted(adm) == sorted(int(ids[j]) for j in expect)
        assert st["admitted"] == len(expect) and st["dropped_overflow"] == len(cand) - len(expect)
        slots = [adm[int(ids[j])] for j in expect]                       # position order -> consecutive slots
        assert slots == [(slots[0] + q) % cap for q in range(len(slots))] if slots else True
        evicted = [int(ids[j]) for j in range(n) if live[j] and look["hit"][j] and not gn[j] < tau]
        assert st["evicted_by_gradient"] == len(evicted) and all(c.map[v] == -1 for v in evicted)
        assert set(before) - set(c.valid_entries(it + 1)) >= set(evicted)


@pytest.mark.parametrize("cap,t_stale,p", [(5, 2, 0.5), (16, 4, 0.9), (40, 50, 0.3)])
def test_without_estimates_and_budget_nothing_changes(cap, t_stale, p):
    """budget None, or a budget of at least the capacity with equal estimates, is the plain rule (dictionary model)."""
    r = np.random.default_rng(cap)
    N = 30
    for kwargs in (dict(), dict(saving=None, budget=cap + 3), dict(saving=np.full(12, 7), budget=cap)):
        c = O.HistoricalCache(N, cap, 3, t_stale)
        m = DictModel(cap, t_stale)
        for i in range(40):
            n = int(r.integers(0, 12))
            ids = r.permutation(N)[:n].astype(np.int32)
            live = r.random(n) < 0.8
            gn = np.round(np.exp(r.standard_normal(n)), 1).astype(np.float32)
            rows = r.standard_normal((n, 3)).astype(np.float32)
            look = O.lookup_prune(c, i, ids, live, None, None, None, 0)
            O.cache_update(c, i, ids, live, look["hit"], gn, p, rows, **kwargs)
            m.update(i, ids, live, gn, p, rows)
            assert set(c.valid_entries(i + 1)) == {v for v in m.where if m.hit(v, i + 1)} and c.head == m.head


def test_iteration_with_budget_admits_the_costliest_rows():
    """Through `iteration`: never more than the budget per layer and update, and when rows are turned away none of them
    has a larger estimate than an admitted one."""
    r = np.random.default_rng(3)
    N, fan, dims = 120, (4, 3, 2), [4, 4, 4, 4]
    g = T.random_explicit_graph(N, 6, 3, allow_isolated=False)
    X = r.standard_normal((N, 4)).astype(np.float32)
    weights = T.random_weights(dims, 3)
    caches = {l: O.HistoricalCache(N, 64, dims[l], 4) for l in (1, 2)}
    budget = {1: 5, 2: 2}
    turned_away = 0
    for it in range(10):
        mb = T.sample(g, r.permutation(N)[:10], fan, it)
        gn = {l: np.exp(r.standard_normal(len(mb.ids[l]))).astype(np.float32) for l in (1, 2)}
        rec = O.iteration(mb, it, caches, lambda ids: X[ids], weights, gn, 0.9, dims, admit_budget=budget)
        for l in (1, 2):
            st = rec["stats"][l]
            assert st["admitted"] <= budget[l]
            turned_away += st["dropped_overflow"]
            adm = admitted_nodes(caches[l], it)
            pos = {int(v): j for j, v in enumerate(mb.ids[l])}
            a = rec["saving"][l]
            cand = [j for j in range(len(mb.ids[l])) if rec["live"][l][j] and not rec["look"][l]["hit"][j] and gn[l][j] < st["tau"]]
            out = [j for j in cand if int(mb.ids[l][j]) not in adm]
            assert len(out) == st["dropped_overflow"]
            if out and adm:
                assert max(a[j] for j in out) <= min(a[pos[v]] for v in adm)
    assert turned_away > 0
