"""Plain CPU statement of the device-side neighbour sampler, used ONLY to check the GPU library: test infrastructure,
never part of the product path. Nothing here is imported by the library or its Python binding, and nothing here
imports them or the input generators.

The paper samples on the CPU (Section 5, the asynchronous sampling threads feeding a task queue) and fixes only the
scheme: uniform neighbour sampling with a fan-out per layer (Section 7.1), from the seeds down to the input layer. What
a sampled mini-batch looks like in memory, which neighbours a fan-out picks and from which random numbers are this
build's reading, stated here in full; the sampler is written with plain Python integers and loops so that it can be
checked against that statement by eye.

Graph: in-neighbour CSR, `indices[indptr[v] : indptr[v + 1]]` are the in-neighbours of v (self loops and repeated
neighbours may occur).

Random numbers: the published SplitMix64 output function as a counter-based generator. word(key, c) =
mix(key + (c + 1) * GAMMA) mod 2**64; the draw of slot j of node v in the block of layer l under mini-batch key K is
word(word(word(mix(K), l), v), j), mapped to [0, 1) by its top 53 bits.

One block (layer l, nodes `cur`, fan-out f), for every node v at position i, with d its degree:
  * d <= f: the candidate slots are 0 .. d-1; otherwise the row is cut into f disjoint strata with integer bounds,
    stratum j = [floor(j d / f), floor((j + 1) d / f)) (each holds at least one slot), draw j (j = 0 .. f-1) picks the
    slot at offset floor(u_j * width_j) of stratum j, and all f slots are then moved round the row by one common
    offset floor(u_f * d) modulo d: f distinct slots for every row, and every slot of the row is taken with
    probability exactly f / d (min(d, f) distinct neighbours when the row has no self loop or repeated neighbour);
  * the candidates are the neighbours at those slots in the order of j, without v itself and without a neighbour that
    already occurred earlier in the same row;
  * the layer below is `cur` followed by the candidates that are not in `cur`, each once, in the order in which they
    first occur (rows in position order, slots in order); the block's columns are positions in that list.
Rows are stored back to back: start[i] = end[i-1], start[0] = 0.

Pins (tests marked "not gpu"): the vectorised input generator of the test harness, which was written separately from
the same statement; membership and stratum of every sampled neighbour; exactly min(d, f) distinct neighbours on
simple graphs; inclusion frequencies against f / d (d not a multiple of f included); the structural invariants of a
mini-batch; published SplitMix64 reference outputs.
"""

MASK = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def mix(x):
    x &= MASK
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & MASK
    return x ^ (x >> 31)


def word(key, counter):
    return mix(key + ((counter & MASK) + 1) * GAMMA)


def unit(w):
    return (w >> 11) * (1.0 / 9007199254740992.0)


def layer_key(key, layer):
    return word(mix(int(key)), int(layer))


def row_candidates(indptr, indices, v, fanout, key_l):
    """The sampled in-neighbours of node v for one block, in slot order."""
    lo, hi = int(indptr[v]), int(indptr[v + 1])
    d = hi - lo
    kv = word(key_l, v)
    out = []
    turn = min(int(unit(word(kv, fanout)) * d), d - 1) if d > fanout else 0
    for j in range(min(d, fanout)):
        if d <= fanout:
            slot = j
        else:
            first, width = (j * d) // fanout, ((j + 1) * d) // fanout - (j * d) // fanout
            slot = (first + min(int(unit(word(kv, j)) * width), width - 1) + turn) % d
        u = int(indices[lo + slot])
        if u != v and u not in out:
            out.append(u)
    return out


def sample_block(indptr, indices, cur, fanout, key_l):
    """One block: returns (start, end, col, col_ids, below) as lists; `below` is the node list of the layer below."""
    below = [int(v) for v in cur]
    where = {v: i for i, v in enumerate(below)}
    assert len(where) == len(below), "the nodes of a layer are distinct"
    start, end, col, col_ids = [], [], [], []
    for v in cur:
        start.append(len(col))
        for u in row_candidates(indptr, indices, int(v), fanout, key_l):
            if u not in where:
                where[u] = len(below)
                below.append(u)
            col.append(where[u])
            col_ids.append(u)
        end.append(len(col))
    return start, end, col, col_ids, below


def sample_minibatch(indptr, indices, seeds, fanouts, key):
    """All blocks from the seed layer L = len(fanouts) down to layer 1 (block l uses fanouts[l - 1]).
    Returns dict(ids=[0..L], start=[..], end=[..], col=[..], col_ids=[..]) with index 0 of the block lists unused."""
    L = len(fanouts)
    ids = [None] * (L + 1)
    start, end, col, col_ids = ([None] * (L + 1) for _ in range(4))
    ids[L] = [int(v) for v in seeds]
    for l in range(L, 0, -1):
        start[l], end[l], col[l], col_ids[l], ids[l - 1] = sample_block(indptr, indices, ids[l], int(fanouts[l - 1]),
                                                                        layer_key(key, l))
    return dict(ids=ids, start=start, end=end, col=col, col_ids=col_ids)


def transpose_block(start, end, col, n_src):
    """The transpose of a sampled block, which the backward pass walks: for every position j of the layer below the rows
    that sampled it, in ascending order, stored back to back. Returns (t_start, t_end, t_row) as lists."""
    rows_of = [[] for _ in range(n_src)]
    for i in range(len(start)):
        for e in range(int(start[i]), int(end[i])):
            rows_of[int(col[e])].append(i)
    t_start, t_end, t_row = [], [], []
    for j in range(n_src):
        t_start.append(len(t_row))
        t_row.extend(rows_of[j])
        t_end.append(len(t_row))
    return t_start, t_end, t_row
