"""Shared test utilities: small explicit graphs, golden-trace parsing, error metrics."""
import os

import numpy as np

from fg_inputs import rng
from fg_inputs.graph import ExplicitGraph
from fg_inputs.sampler import sample_minibatch

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def random_explicit_graph(num_nodes, max_deg, seed, allow_isolated=True):
    """In-neighbour CSR without self loops or parallel edges; degrees in [0 or 1, max_deg]."""
    r = np.random.default_rng(seed)
    indptr = [0]
    indices = []
    for v in range(num_nodes):
        d = int(r.integers(0 if allow_isolated else 1, max_deg + 1))
        cand = r.permutation(num_nodes)
        nb = [int(u) for u in cand if u != v][:d]
        indices.extend(nb)
        indptr.append(len(indices))
    return ExplicitGraph(np.array(indptr), np.array(indices, dtype=np.int64))


def dense_adjacency(g):
    n = g.num_nodes
    A = np.zeros((n, n), dtype=np.float64)
    for v in range(n):
        A[v, g.indices[g.indptr[v]:g.indptr[v + 1]]] = 1.0
    return A


def random_weights(dims, seed, scale=None):
    r = np.random.default_rng(seed)
    out = {}
    for l in range(1, len(dims)):
        d_in, d_out = dims[l - 1], dims[l]
        W = (r.standard_normal((2 * d_in, d_out)) / np.sqrt(2 * d_in)).astype(np.float32)
        b = (0.1 * r.standard_normal(d_out)).astype(np.float32)
        out[l] = (W, b)
    return out


def sample(g, seeds, fanouts, it, seed=7):
    return sample_minibatch(g, np.asarray(seeds), fanouts, rng.make_key(seed, it))


def parse_trace(name):
    """Parse a hand-worked cache trace from tests/golden (format described in the file's header)."""
    params, steps = {}, []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.rstrip("\n")
        if not line.strip() or line.lstrip().startswith("#"):
            continue
        if not line.startswith("iter"):
            k, v = line.split()
            params[k] = float(v) if "." in v else int(v)
            continue
        fields = [f.strip() for f in line.split("|")]
        step = dict(iter=int(fields[0].split()[1]))
        for f in fields[1:]:
            toks = f.split()
            key, vals = toks[0], toks[1:]
            if key == "live":
                step["live"] = [(int(t.split(":")[0]), float(t.split(":")[1])) for t in vals]
            elif key == "hits":
                step["hits"] = [int(t) for t in vals]
            elif key == "valid_after":
                step["valid_after"] = {int(t.split("@")[0]): int(t.split("@")[1]) for t in vals}
            elif key == "slots":
                step["slots"] = [int(t) for t in vals]
            elif key == "head":
                step["head"] = int(vals[0])
        steps.append(step)
    return params, steps


def rel_err_rows(got, ref):
    """Max over elements of |got-ref| / max(|ref|, rowmax(|ref|)/16); rows whose reference is all zero must be zero.

    "Relative error" is undefined at a zero reference element (half of a ReLU output), so the
    denominator is floored at 1/16 of the row's largest magnitude.
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rowmax = np.abs(ref).max(axis=1, keepdims=True)
    zero_rows = (rowmax[:, 0] == 0)
    if zero_rows.any() and np.abs(got[zero_rows]).max() != 0:
        return np.inf
    den = np.maximum(np.abs(ref), rowmax / 16.0)
    den[zero_rows] = 1.0
    return float((np.abs(got - ref) / den).max())
