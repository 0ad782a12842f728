"""Pins of the oracle's neighbour sampler (no GPU): published SplitMix64 outputs, the separately written vectorised
sampler of the test harness, and what the stated scheme implies for every sampled neighbour."""
import numpy as np
import pytest

from fg_inputs import rng
from oracle import sampler_oracle as S
from tests import helpers as T


def multigraph(num_nodes, max_deg, seed):
    """In-neighbour CSR whose rows are drawn with replacement from a few nodes around v, v included: self loops and
    repeated neighbours are common."""
    from fg_inputs.graph import ExplicitGraph
    r = np.random.default_rng(seed)
    indptr, indices = [0], []
    for v in range(num_nodes):
        d = int(r.integers(0, max_deg + 1))
        indices.extend(((v + r.integers(-3, 4, size=d)) % num_nodes).tolist())
        indptr.append(len(indices))
    return ExplicitGraph(np.array(indptr), np.array(indices, dtype=np.int64))


def test_generator_reproduces_published_splitmix64_outputs():
    # the first three outputs of SplitMix64 seeded with 0 (reference implementation by Vigna, splitmix64.c)
    assert [S.word(0, c) for c in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert 0.0 <= S.unit(S.word(5, 7)) < 1.0 and S.unit((1 << 64) - 1) == 1.0 - 2.0 ** -53 and S.unit(0) == 0.0


@pytest.mark.parametrize("seed,fanouts,max_deg", [(0, (3, 2), 6), (1, (4, 3, 2), 9), (2, (2, 2, 2, 2), 5), (3, (10, 5), 40)])
def test_matches_the_vectorised_harness_sampler(seed, fanouts, max_deg):
    N = 120
    g = T.random_explicit_graph(N, max_deg, seed) if seed % 2 == 0 else multigraph(N, max_deg, seed)
    r = np.random.default_rng(seed)
    for it in range(4):
        seeds = r.permutation(N)[:9]
        key = int(rng.make_key(seed, it))
        mb = T.sample(g, seeds, fanouts, it, seed=seed)
        got = S.sample_minibatch(g.indptr, g.indices, seeds, fanouts, int(rng.make_key(seed, it)))
        L = len(fanouts)
        for l in range(L + 1):
            assert got["ids"][l] == mb.ids[l].tolist()
        for l in range(1, L + 1):
            assert got["start"][l] == mb.start[l].tolist() and got["end"][l] == mb.end[l].tolist()
            assert got["col"][l] == mb.col[l].tolist()
            assert got["col_ids"][l] == mb.ids[l - 1][mb.col[l]].tolist()
        assert key == int(rng.make_key(seed, it))


def test_every_sampled_neighbour_is_a_neighbour_from_its_own_stratum():
    g = multigraph(200, 60, 5)
    f = 7
    key_l = S.layer_key(99, 2)
    for v in range(200):
        nb = g.indices[g.indptr[v]:g.indptr[v + 1]].tolist()
        d = len(nb)
        got = S.row_candidates(g.indptr, g.indices, v, f, key_l)
        assert len(set(got)) == len(got) and v not in got and set(got) <= set(nb)
        if d <= f:
            assert got == list(dict.fromkeys(u for u in nb if u != v))          # all of them, in slot order, once each
        else:
            # stratum j holds the slots [floor(j d / f), floor((j + 1) d / f)), all moved round the row by one offset:
            # for some offset every candidate must come from a stratum of its own, in the order of j
            def reachable(turn):
                strata = [{nb[(s + turn) % d] for s in range(j * d // f, (j + 1) * d // f)} for j in range(f)]
                j = 0
                for u in got:
                    while j < f and u not in strata[j]:
                        j += 1
                    if j == f:
                        return False
                    j += 1
                return True
            assert any(reachable(t) for t in range(d))


@pytest.mark.parametrize("f", [3, 5, 10, 15])
def test_a_row_without_self_loop_or_repeats_gets_exactly_min_degree_fanout_distinct_neighbours(f):
    """Section 7.1: a fan-out of f samples f neighbours of a node that has more than f; all of them otherwise."""
    g = T.random_explicit_graph(150, 40, 11 + f, allow_isolated=True)       # simple graph: no self loops, no parallel edges
    key_l = S.layer_key(5, 1)
    deg = np.diff(g.indptr)
    assert (deg > f).sum() > 20 and ((deg % f != 0) & (deg > f)).sum() > 10
    for v in range(150):
        got = S.row_candidates(g.indptr, g.indices, v, f, key_l)
        assert len(got) == len(set(got)) == min(int(deg[v]), f), (v, int(deg[v]), got)
    out = S.sample_minibatch(g.indptr, g.indices, list(range(0, 150, 3)), (f, f), 77)
    for l in (1, 2):
        want = np.minimum(deg[np.array(out["ids"][l])], f)
        assert (np.array(out["end"][l]) - np.array(out["start"][l])).tolist() == want.tolist()


@pytest.mark.parametrize("d,f", [(12, 4), (13, 4), (7, 5), (50, 15)])
def test_inclusion_frequencies_are_uniform(d, f):
    """A node with d distinct neighbours and fan-out f: over many keys every neighbour is sampled f/d of the time,
    also when f does not divide d."""
    indptr = np.array([0, d] + [d] * d)
    indices = np.arange(1, d + 1)
    count = np.zeros(d + 1)
    trials = 6000
    for k in range(trials):
        got = S.row_candidates(indptr, indices, 0, f, S.layer_key(k, 1))
        assert len(got) == f
        for u in got:
            count[u] += 1
    freq = count[1:] / trials
    p = f / d
    assert np.all(np.abs(freq - p) < 5 * np.sqrt(p * (1 - p) / trials)), freq


def test_minibatch_structure():
    g = T.random_explicit_graph(300, 12, 8)
    out = S.sample_minibatch(g.indptr, g.indices, list(range(0, 40, 2)), (5, 4, 3), 1234)
    L = 3
    for l in range(L + 1):
        assert len(set(out["ids"][l])) == len(out["ids"][l])
    for l in range(1, L + 1):
        n = len(out["ids"][l])
        assert out["ids"][l - 1][:n] == out["ids"][l]
        assert out["start"][l][0] == 0 and out["start"][l][1:] == out["end"][l][:-1] and out["end"][l][-1] == len(out["col"][l])
        assert [out["ids"][l - 1][c] for c in out["col"][l]] == out["col_ids"][l]
        # new nodes appear in order of first occurrence
        firsts = list(dict.fromkeys(u for u in out["col_ids"][l] if u not in set(out["ids"][l])))
        assert out["ids"][l - 1][n:] == firsts
    # different layers of one mini-batch draw from different streams
    assert S.layer_key(1234, 1) != S.layer_key(1234, 2)


def test_transpose_lists_every_edge_once_under_its_source():
    """Against the harness's sort-based transpose (written separately) and against the definition edge by edge, on blocks
    with pruned rows in between."""
    from fg_inputs.sampler import transpose_block
    g = multigraph(300, 20, 9)
    out = S.sample_minibatch(g.indptr, g.indices, list(range(0, 120, 3)), (6, 4), 77)
    for l in (1, 2):
        start, end, col = np.array(out["start"][l]), np.array(out["end"][l]), np.array(out["col"][l])
        end = np.where(np.arange(len(end)) % 5 == 2, start, end)                 # some rows pruned
        n_src = len(out["ids"][l - 1])
        ts, te, tr = S.transpose_block(start, end, col, n_src)
        hs, he, hr = transpose_block(start, end, col, n_src)
        assert ts == hs.tolist() and te == he.tolist() and tr == hr.tolist()
        edges = sorted((int(col[e]), i) for i in range(len(start)) for e in range(start[i], end[i]))
        assert [(j, r) for j in range(n_src) for r in tr[ts[j]:te[j]]] == edges
        assert ts[0] == 0 and ts[1:] == te[:-1] and te[-1] == len(edges)


def test_transpose_hand_example():
    """Three rows over four sources: row 0 samples positions 1, 0; row 1 nothing; row 2 samples positions 1, 2."""
    ts, te, tr = S.transpose_block([0, 2, 2], [2, 2, 4], [1, 0, 1, 2], 4)
    assert (ts, te, tr) == ([0, 1, 3, 4], [1, 3, 4, 4], [0, 0, 2, 2])
    # a pruned row (end = start) drops out; the column array keeps its entries
    ts, te, tr = S.transpose_block([0, 2, 2], [0, 2, 4], [1, 0, 1, 2], 4)
    assert (ts, te, tr) == ([0, 0, 1, 2], [0, 1, 2, 2], [2, 2])


# ---------------------------------------------------------------- do these pins bite?

SAMPLER_MUTANTS = [
    ("self loops are kept", "row_candidates", "if u != v and u not in out:", "if u not in out:"),
    ("repeated neighbours are kept", "row_candidates", "if u != v and u not in out:", "if u != v:"),
    ("every stratum is sampled at its first slot", "row_candidates", "min(int(unit(word(kv, j)) * width), width - 1)", "0"),
    ("slots are drawn from the whole row", "row_candidates", "first + min(int(unit(word(kv, j)) * width), width - 1)", "int(unit(word(kv, j)) * d)"),
    ("strata have real-valued bounds, so neighbouring ones share a slot", "row_candidates",
     "slot = (first + min(int(unit(word(kv, j)) * width), width - 1) + turn) % d", "slot = (min(int((j + unit(word(kv, j))) * (d / fanout)), d - 1) + turn) % d"),
    ("the choice is not turned round the row", "row_candidates", "turn = min(int(unit(word(kv, fanout)) * d), d - 1) if d > fanout else 0", "turn = 0"),
    ("the turn shares its draw with the first stratum", "row_candidates", "unit(word(kv, fanout)) * d", "unit(word(kv, 0)) * d"),
    ("the last stratum stops one slot early", "row_candidates", "((j + 1) * d) // fanout - (j * d) // fanout", "max(((j + 1) * d) // fanout - (j * d) // fanout - (1 if j == fanout - 1 else 0), 1)"),
    ("the slot's draw ignores the node", "row_candidates", "kv = word(key_l, v)", "kv = key_l"),
    ("all slots of a node share one draw", "row_candidates", "unit(word(kv, j))", "unit(word(kv, 0))"),
    ("small rows lose their last neighbour", "row_candidates", "range(min(d, fanout))", "range(min(d, fanout) - (1 if d <= fanout and d > 1 else 0))"),
    ("new nodes are numbered from zero", "sample_block", "where[u] = len(below)", "where[u] = len(below) - len(cur)"),
    ("every occurrence appends a node", "sample_block", "if u not in where:", "if True:"),
    ("layers share their stream", "layer_key", "return word(mix(int(key)), int(layer))", "return word(mix(int(key)), 0)"),
    ("the key is used unmixed", "layer_key", "word(mix(int(key)), int(layer))", "word(int(key), int(layer))"),
    ("rows are not stored back to back", "sample_block", "start.append(len(col))", "start.append(len(col) + (1 if col else 0))"),
    ("the generator drops its second round", "mix", "x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & MASK", "pass"),
    ("the top bits are not the ones used", "unit", "(w >> 11)", "(w & ((1 << 53) - 1))"),
    ("the transpose files an edge under its row", "transpose_block", "rows_of[int(col[e])].append(i)", "rows_of[i % n_src].append(int(col[e]))"),
    ("the transpose lists of consecutive sources overlap", "transpose_block", "t_start.append(len(t_row))", "t_start.append(max(len(t_row) - 1, 0))"),
]

SAMPLER_PINS = [
    (test_generator_reproduces_published_splitmix64_outputs, [()]),
    (test_matches_the_vectorised_harness_sampler, [(0, (3, 2), 6), (1, (4, 3, 2), 9), (3, (10, 5), 40)]),
    (test_every_sampled_neighbour_is_a_neighbour_from_its_own_stratum, [()]),
    (test_a_row_without_self_loop_or_repeats_gets_exactly_min_degree_fanout_distinct_neighbours, [(3,), (10,)]),
    (test_inclusion_frequencies_are_uniform, [(12, 4), (13, 4)]),
    (test_minibatch_structure, [()]),
    (test_transpose_lists_every_edge_once_under_its_source, [()]),
    (test_transpose_hand_example, [()]),
]


@pytest.mark.parametrize("what,name,old,new", SAMPLER_MUTANTS, ids=[m[0] for m in SAMPLER_MUTANTS])
def test_a_planted_mistake_in_the_sampler_fails_a_pin(what, name, old, new):
    import inspect
    import textwrap
    original = getattr(S, name)
    src = textwrap.dedent(inspect.getsource(original))
    assert src.count(old) == 1, f"the text to change occurs {src.count(old)} times in {name}"
    scope = {}
    exec(compile(src.replace(old, new), f"<mutant of {name}>", "exec"), S.__dict__, scope)
    setattr(S, name, scope[name])
    caught = None
    try:
        for fn, cases in SAMPLER_PINS:
            for args in cases:
                try:
                    fn(*args)
                except Exception as e:
                    caught = f"{fn.__name__}: {type(e).__name__}"
                    break
            if caught:
                break
    finally:
        setattr(S, name, original)
    assert caught is not None, f"no pin notices that {what}"
