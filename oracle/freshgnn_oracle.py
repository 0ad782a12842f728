"""Plain CPU statement of one training iteration's data path with a selective
historical-embedding cache (Algorithm 1 of the paper), used ONLY to check the
GPU library: test infrastructure, never part of the product path. Nothing here
is imported by the library or its Python binding, and nothing here imports them.

The method is an approximation scheme (Eq. 2: cached embeddings stand in for
recomputed ones), so this file is the algorithm itself, step by step, in the
paper's order and notation, with floating point carried in float64 and rounded
once to the storage type:

  top-down   (Alg. 1, the lookup / remove_subgraph / V_normal lines): `lookup_prune`
  loader     (Alg. 1, Load_feature line; Section 6, one-sided reads): `gather`
  bottom-up  (Alg. 1, the cache fetch line and the f_W line; Eq. 1): `gather`,
             `aggregate`, `linear`
  update     (Alg. 1, Update line; Sections 4.1.1, 4.1.2, 4.2): `cache_update`
  feature side of the bidirectional cache (Section 4.2): `BidirectionalCache`, `hot_order`;
             `iteration(..., feature_side=...)` loads raw features through it
  backward   (Alg. 1, the loss and loss.backward() lines; Section 4.1.1: the embedding gradients whose norms
             drive admission and check-out): `softmax_xent_grad`, `layer_backward`, `row_norms`, `backward`;
             `iteration(..., labels=...)` takes the gradient norms from it instead of from the caller
  access-aware admission (Section 7.4 names a policy that prefers embeddings saving more memory access, without
             a rule): `access_estimate`, `cache_update(..., saving=, budget=)`, `iteration(..., admit_budget=...)`

Where the paper leaves something open (the Update procedure has no printed body;
mini-batch layout; percentile ties; slot capacity) the reading taken is stated in
the docstring of the function concerned.

Pins (tests marked "not gpu"): dense whole-graph recursion of Eq. 1 on small
graphs with full neighbourhoods; closed forms of the mean; identity-panel
weights; a depth-first "needed set" for the pruning; a dictionary model of the
cache; hand-worked admit/evict/staleness/ring traces; the degenerate settings of
Section 4.1.3; for the shared buffer a byte-by-byte model of what has been overwritten,
a hand-worked displacement trace, and the bit-identity of every loaded feature row; for the backward
pass (GraphSAGE and GCN layers) central finite differences of the loss through the forward functions of this file;
for the mixed-precision setting (fp16 features, bf16 operands of every matrix product, bf16 embeddings, fp32 last
layer) a hand-worked example, identity-panel weights that expose each rounded operand bit for bit, and exact
rational arithmetic, with a library bfloat16 conversion as the rounding routine. The I/O-saving percentages the paper reports depend on its
datasets and real gradients: parity unpinned for those, they are not reproduced.
The access-aware admission is pinned to the reading stated in `access_estimate` and `cache_update` (an
instrumented recursive evaluation that counts the rows it reads, closed forms on full trees, the rank definition
of "the B largest", the dictionary model); against the paper it is parity unpinned: the paper gives no rule.
"""
import numpy as np

FLOAT_TYPES = ("f32", "f16", "bf16")


# --------------------------------------------------------------------------- storage types

def round_bf16(x):
    """Round to the nearest bfloat16 (ties to even); result held in float32."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    b = x32.view(np.uint32).astype(np.uint64)
    r = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return r.astype(np.uint32).view(np.float32).reshape(x32.shape)


def round_to(x, dtype):
    """Round float64 values once to storage type `dtype`; bf16 is held as float32 values."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "f16":
        return np.asarray(x, dtype=np.float64).astype(np.float16)
    if dtype == "bf16":
        # float64 -> float32 -> bf16 double rounding matches a device that converts an fp32 result
        return round_bf16(x)
    raise ValueError(dtype)


def storage_numpy_dtype(dtype):
    return {"f32": np.float32, "f16": np.float16, "bf16": np.float32}[dtype]


def element_bytes(dtype):
    return {"f32": 4, "f16": 2, "bf16": 2}[dtype]


def row_image(values, dtype):
    """The bytes a row of storage type `dtype` occupies in memory (little endian); bf16 = upper half of the fp32 word."""
    if dtype == "f32":
        return np.ascontiguousarray(values, dtype=np.float32).view(np.uint8)
    if dtype == "f16":
        return np.ascontiguousarray(values, dtype=np.float16).view(np.uint8)
    if dtype == "bf16":
        bits = np.ascontiguousarray(values, dtype=np.float32).view(np.uint32) >> np.uint32(16)
        return bits.astype(np.uint16).view(np.uint8)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- the cache C^(l)

class HistoricalCache:
    """Historical embedding cache of one layer (Section 4.2, embedding side).

    State, following the paper's description: a node-id mapping array of length |V| whose
    entry is the slot holding that node's embedding (or -1), a slot table of embeddings, and a
    ring header that moves forward as embeddings are admitted. Per slot this model also keeps
    the owning node and the iteration that admitted it ("auxiliary data related to staleness").

    Reading taken for staleness (Section 4.1.2): an embedding admitted by the update of
    iteration a has staleness i - a when looked up in iteration i; it is usable while
    1 <= i - a <= t_stale, so t_stale = 0 disables the cache (Section 4.1.3). The paper's
    implementation note that the header is reset every t_stale iterations is replaced by a
    per-slot stamp with a modulo ring: the oldest slots are overwritten first and the bound
    is exact.
    """

    def __init__(self, num_nodes, capacity, dim, t_stale, dtype="f32", storage=None):
        """`storage`: optional uint8 array of capacity * dim * element_bytes bytes in which every admitted row is
        also laid down byte for byte (slot s at s * row bytes): the ring's share of a buffer it has in common
        with raw features (`BidirectionalCache`)."""
        self.num_nodes = int(num_nodes)
        self.capacity = int(capacity)
        self.dim = int(dim)
        self.t_stale = int(t_stale)
        self.dtype = dtype
        self.map = np.full(self.num_nodes, -1, dtype=np.int32)
        self.slot_node = np.full(self.capacity, -1, dtype=np.int32)
        self.slot_stamp = np.zeros(self.capacity, dtype=np.int32)
        self.table = np.zeros((self.capacity, self.dim), dtype=storage_numpy_dtype(dtype))
        self.head = 0
        self.used = 0            # slots written at least once: 0 .. used-1 (the ring fills upwards until it first wraps)
        self.storage = storage
        self.row_bytes = self.dim * element_bytes(dtype)
        if storage is not None:
            assert storage.dtype == np.uint8 and storage.shape == (self.capacity * self.row_bytes,)

    def store(self, s, row):
        """Write an embedding into slot s (the table and, if the ring lives in a shared buffer, its bytes there)."""
        self.table[s] = row
        if self.storage is not None:
            self.storage[s * self.row_bytes:(s + 1) * self.row_bytes] = row_image(self.table[s], self.dtype)

    def slot_of(self, v, i):
        """Slot holding a usable embedding of node v at iteration i, or -1 (the set C^(l) is {v: slot_of >= 0})."""
        s = int(self.map[v])
        if s < 0:
            return -1
        if int(self.slot_node[s]) != int(v):
            return -1          # the slot has been recycled for another node
        age = int(i) - int(self.slot_stamp[s])
        if age < 1 or age > self.t_stale:
            return -1
        return s

    def valid_entries(self, i):
        """{node: (slot, stamp)} of everything a lookup at iteration i would hit."""
        out = {}
        for s in range(self.capacity):
            v = int(self.slot_node[s])
            if v >= 0 and self.slot_of(v, i) == s:
                out[v] = (s, int(self.slot_stamp[s]))
        return out


# --------------------------------------------------------------------------- feature side (Section 4.2)

RING_ALIGN = 256   # a ring's first byte in the shared buffer is rounded up to this


def hot_order(score, count):
    """The `count` nodes with the largest estimated saved memory access, largest first (ties: smaller id first).

    The paper orders the raw features it caches by that estimate without defining it; `score[v]` is whatever
    estimate the caller has (the tests and workloads use how often v is named as a neighbour).
    """
    score = np.asarray(score, dtype=np.float64)
    order = sorted(range(len(score)), key=lambda v: (-score[v], v))
    return np.asarray(order[:int(count)], dtype=np.int32)


class BidirectionalCache:
    """The device buffer that raw features and historical embeddings share (Section 4.2, "bidirectional cache").

    One buffer of `buffer_bytes` bytes.
      * Embedding side, from the left end: the ring of cached layer 1, then layer 2, ...; a ring starts at the
        next multiple of RING_ALIGN and slot s of ring l occupies the bytes [base_l + s*row_l, base_l + (s+1)*row_l).
        The rings are `HistoricalCache` objects that lay their admitted rows down in this buffer.
      * Feature side, from the right end: before training the raw feature rows of the hot nodes are written, the
        one of rank r (0 = largest estimated saved access) at [B - (r+1)*w, B - r*w), w = bytes of a feature row.
        The more valuable a row, the farther it is from the embeddings.
      * Junction: the two sides may overlap. A feature row is lost the moment an embedding is written over any of
        its bytes, and not earlier. A ring hands out slots 0, 1, 2, ... until it first wraps, so the bytes ring l
        has written are exactly [base_l, base_l + used_l*row_l).
    Reading taken where the paper is silent: one ring per cached layer with the preset capacity (the rings do not
    grow past it), laid out in layer order; a feature row straddling the end of a ring's written part counts as lost.
    """

    def __init__(self, num_nodes, capacities, dims, t_stale, dtype, buffer_bytes):
        self.num_nodes = int(num_nodes)
        self.buffer_bytes = int(buffer_bytes)
        self.buf = np.zeros(self.buffer_bytes, dtype=np.uint8)
        self.rings = {}
        self.ring_base = {}
        at = 0
        for k, (cap, dim) in enumerate(zip(capacities, dims)):
            l = k + 1
            at = -(-at // RING_ALIGN) * RING_ALIGN
            size = int(cap) * int(dim) * element_bytes(dtype)
            assert at + size <= self.buffer_bytes, "the rings do not fit into the buffer"
            self.ring_base[l] = at
            self.rings[l] = HistoricalCache(num_nodes, cap, dim, t_stale, dtype, storage=self.buf[at:at + size])
            at += size
        self.rank_of = np.full(self.num_nodes, -1, dtype=np.int32)   # node -> rank of its row on the feature side
        self.n_feat = 0
        self.feat_row_bytes = 0
        self.feat_dtype = None

    def fill_features(self, hot_ids, feature_rows, feat_dtype):
        """Populate the buffer with the rows of `hot_ids` (hottest first, distinct) before any embedding is admitted."""
        assert all(r.used == 0 for r in self.rings.values()), "features are placed before training starts"
        hot_ids = np.asarray(hot_ids, dtype=np.int64)
        assert len(np.unique(hot_ids)) == len(hot_ids)
        rows = np.asarray(feature_rows(hot_ids))
        w = rows.shape[1] * element_bytes(feat_dtype) if len(hot_ids) else 0
        assert len(hot_ids) * w <= self.buffer_bytes, "more rows than the buffer holds"
        self.rank_of[:] = -1
        self.n_feat, self.feat_row_bytes, self.feat_dtype = len(hot_ids), w, feat_dtype
        B = self.buffer_bytes
        for r, v in enumerate(hot_ids):
            self.buf[B - (r + 1) * w:B - r * w] = row_image(rows[r], feat_dtype)
            self.rank_of[v] = r

    def feature_rank(self, v):
        """Rank of node v's row if it is on the feature side and no embedding has been written over it, else -1."""
        r = int(self.rank_of[v])
        if r < 0:
            return -1
        lo = self.buffer_bytes - (r + 1) * self.feat_row_bytes
        hi = lo + self.feat_row_bytes
        for l, ring in self.rings.items():
            w_lo = self.ring_base[l]
            w_hi = w_lo + ring.used * ring.row_bytes
            if ring.used > 0 and lo < w_hi and hi > w_lo:   # overlap with a non-empty written range
                return -1
        return r

    def load(self, ids, feature_rows):
        """Load_feature through the feature side: rows of `ids`, those still cached taken from the buffer, the rest
        from the table. Returns (rows, from_buffer flags); the rows are bit copies either way."""
        ids = np.asarray(ids, dtype=np.int64)
        ranks = np.asarray([self.feature_rank(v) for v in ids], dtype=np.int64)
        miss = ranks < 0
        if miss.all():
            return np.asarray(feature_rows(ids)), ~miss
        B, w = self.buffer_bytes, self.feat_row_bytes
        np_dt = storage_numpy_dtype(self.feat_dtype)
        out = np.zeros((len(ids), w // element_bytes(self.feat_dtype)), dtype=np_dt)
        if miss.any():
            out[miss] = feature_rows(ids[miss])
        for k in np.nonzero(~miss)[0]:
            r = ranks[k]
            out[k] = self.buf[B - (r + 1) * w:B - r * w].view(np_dt)
        return out, ~miss


# --------------------------------------------------------------------------- top-down pass

def lookup_prune(cache, i, ids, live, start, end, col, n_src):
    """One layer of the top-down pass (Alg. 1: V_cache = V ∩ C, remove_subgraph, V_normal = V \\ V_cache).

    ids     node ids of layer l, by position
    live    bool per position: still needed after pruning the layers above (None: all)
    start, end, col   block l in the two-row-array format of Section 5 (None for layer 0);
            `end` is modified in place: rows that are not normal get end = start
    n_src   number of positions in layer l-1

    A node is looked up only if it is live (a pruned node is no longer part of G_b). Hits form
    V_cache; live non-hits form V_normal. The neighbours that remain needed in layer l-1 are
    the normal rows themselves (their own previous embedding) and their sampled neighbours:
    that is what removing the subgraph below every hit leaves.

    Returns hit (bool[n]), hit_pos, hit_slot, normal_pos (ascending positions) and
    live_src (bool[n_src], None without a block).
    """
    n = len(ids)
    live = np.ones(n, dtype=bool) if live is None else np.asarray(live, dtype=bool)
    hit = np.zeros(n, dtype=bool)
    hit_pos, hit_slot, normal_pos = [], [], []
    for j in range(n):
        if not live[j]:
            continue
        s = cache.slot_of(int(ids[j]), i) if cache is not None else -1
        if s >= 0:
            hit[j] = True
            hit_pos.append(j)
            hit_slot.append(s)
        else:
            normal_pos.append(j)
    live_src = None
    if start is not None:
        live_src = np.zeros(n_src, dtype=bool)
        normal = live & ~hit
        for j in range(n):
            if normal[j]:
                live_src[j] = True
                live_src[col[start[j]:end[j]]] = True
            else:
                end[j] = start[j]
    return dict(hit=hit, hit_pos=np.asarray(hit_pos, dtype=np.int32), hit_slot=np.asarray(hit_slot, dtype=np.int32),
                normal_pos=np.asarray(normal_pos, dtype=np.int32), live_src=live_src,
                counts=(int(live.sum()), len(hit_pos), len(normal_pos)))


# --------------------------------------------------------------------------- loader / cache fetch

def gather(table_rows, index, dst, dst_pos=None):
    """dst[dst_pos[k], :] = table[index[k], :], a bit copy (Load_feature, and the C^(l)[v] fetch).

    `table_rows(index_array)` returns the rows; dst_pos None means k itself.
    """
    index = np.asarray(index)
    rows = table_rows(index)
    if dst_pos is None:
        dst[:len(index)] = rows
    else:
        dst[np.asarray(dst_pos)] = rows
    return dst


# --------------------------------------------------------------------------- one GNN layer (Eq. 1, GraphSAGE mean)

def aggregate(start, end, col, rows, h_src):
    """Mean of the sampled neighbours' previous-layer rows, per row in `rows`: float64 [len(rows), d].

    AGG of Eq. 1 with the mean aggregator; a row without neighbours gets the zero vector.
    """
    h = np.asarray(h_src)
    out = np.zeros((len(rows), h.shape[1]), dtype=np.float64)
    for k, r in enumerate(rows):
        nb = col[start[r]:end[r]]
        if len(nb):
            out[k] = h[nb].astype(np.float64).sum(axis=0) / float(len(nb))
    return out


def linear(h_self, agg, W, b, relu):
    """phi of Eq. 1 for GraphSAGE-mean: act([h_self ‖ agg] · W + b) in float64.

    W is [2*d_in, d_out]; its first d_in rows multiply the node's own previous embedding, the
    last d_in rows the neighbour mean. ReLU between layers, identity after the last.
    """
    d_in = h_self.shape[1]
    W = np.asarray(W, dtype=np.float64)
    z = (np.asarray(h_self, dtype=np.float64) @ W[:d_in] + np.asarray(agg, dtype=np.float64) @ W[d_in:]
         + np.asarray(b, dtype=np.float64))
    return np.maximum(z, 0.0) if relu else z


def aggregate_gcn(start, end, col, rows, h_src):
    """Propagation of a GCN layer in its row-normalised form, per row in `rows`: the mean over the row's own previous
    embedding and those of its sampled neighbours, (h_v + sum_u h_u) / (deg + 1): float64 [len(rows), d].

    The paper names GCN among its models without writing the layer down. The graph convolution adds a self loop and
    normalises by degree; on a sampled block only the row's own sampled degree is known, so the normalisation is by
    row (the mean aggregator with the node itself included), followed by one weight matrix (`linear_gcn`).
    """
    h = np.asarray(h_src)
    out = np.zeros((len(rows), h.shape[1]), dtype=np.float64)
    for k, r in enumerate(rows):
        nb = col[start[r]:end[r]]
        out[k] = (h[r].astype(np.float64) + h[nb].astype(np.float64).sum(axis=0)) / float(len(nb) + 1)
    return out


def linear_gcn(agg, W, b, relu):
    """act(agg · W + b) with W [d_in, d_out]: the dense part of a GCN layer, float64."""
    z = np.asarray(agg, dtype=np.float64) @ np.asarray(W, dtype=np.float64) + np.asarray(b, dtype=np.float64)
    return np.maximum(z, 0.0) if relu else z


# --------------------------------------------------------------------------- loss and backward pass

def softmax_xent(h, labels):
    """Mean softmax cross-entropy of the seed outputs (the loss line of Alg. 1; the paper does not fix the loss,
    node classification is its task): L = -(1/n) sum_i log softmax(h_i)[label_i], in float64."""
    h = np.asarray(h, dtype=np.float64)
    z = h - h.max(axis=1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=1, keepdims=True))
    return float(-logp[np.arange(len(h)), np.asarray(labels)].mean()) if len(h) else 0.0


def softmax_xent_grad(h, labels):
    """dL/dh for `softmax_xent`: (softmax(h_i) - onehot(label_i)) / n, float64 [n, d]."""
    h = np.asarray(h, dtype=np.float64)
    if len(h) == 0:
        return np.zeros_like(h)
    z = h - h.max(axis=1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(len(h)), np.asarray(labels)] -= 1.0
    return p / len(h)


def row_norms(x):
    """L2 norm of every row (the "magnitude of embedding gradients" of Section 4.1.1), float64."""
    x = np.asarray(x, dtype=np.float64)
    return np.sqrt((x * x).sum(axis=1))


def layer_backward(start, end, col, rows, dh, h_out, h_self, agg, W, n_src, relu, compute_dtype="f32"):
    """Backward of one GraphSAGE-mean layer (Eq. 1 with the readings of `aggregate` and `linear`) for the rows in
    `rows` (V_normal of the layer; fetched and pruned rows were not computed, so nothing flows below them).

    dh      dL/dH(l) by position [n_l, d_out]      h_out  H(l) by position (ReLU passes gradient where it is > 0)
    h_self  H(l-1)[rows], agg = the means that entered the layer, both [len(rows), d_in]
    Returns dL/dH(l-1) by position [n_src, d_in], dL/dW [2*d_in, d_out], dL/db [d_out], all float64:
      dz = dh[rows] * (h_out[rows] > 0)  (no mask after the last layer)
      dW = [h_self ‖ agg]^T dz,  db = sum of dz,  [d_self ‖ d_agg] = dz W^T
      dH(l-1)[r] += d_self  for r in rows;  dH(l-1)[c] += d_agg / deg(r)  for every sampled neighbour c of r
    In the bf16 setting the operands of both matrix products are bf16, as in the forward product: dz is rounded to
    bf16 before it enters dz W^T and [h_self ‖ agg]^T dz (h_self and agg arrive rounded, W is rounded here); the bias
    gradient sums the unrounded dz; products, sums and every result stay in higher precision.
    """
    W = np.asarray(W, dtype=np.float64)
    d_in = W.shape[0] // 2
    dz = np.asarray(dh, dtype=np.float64)[rows]
    if relu:
        dz = dz * (np.asarray(h_out)[rows] > 0)
    db = dz.sum(axis=0)
    if compute_dtype == "bf16":
        dz = round_bf16(dz).astype(np.float64)
        W = round_bf16(W).astype(np.float64)
    x = np.concatenate([np.asarray(h_self, dtype=np.float64), np.asarray(agg, dtype=np.float64)], axis=1)
    dW = x.T @ dz
    dx = dz @ W.T
    dsrc = np.zeros((n_src, d_in), dtype=np.float64)
    for k, r in enumerate(rows):
        dsrc[r] += dx[k, :d_in]
        nb = col[start[r]:end[r]]
        if len(nb):
            np.add.at(dsrc, nb, dx[k, d_in:] / float(len(nb)))
    return dsrc, dW, db


def layer_backward_gcn(start, end, col, rows, dh, h_out, agg, W, n_src, relu):
    """Backward of one GCN layer in the form of `aggregate_gcn` / `linear_gcn`, for the rows in `rows`.

    agg = the propagated rows m_r = (h_r + sum of the sampled neighbours' rows) / (deg(r) + 1) that entered the layer.
      dz = dh[rows] * (h_out[rows] > 0)  (no mask after the last layer)
      dW = agg^T dz,  db = sum of dz,  dm = dz W^T
      dH(l-1)[r] += dm_r / (deg(r) + 1);  dH(l-1)[c] += dm_r / (deg(r) + 1)  for every sampled neighbour c of r
    Returns dL/dH(l-1) by position [n_src, d_in], dL/dW [d_in, d_out], dL/db [d_out], float64.
    """
    W = np.asarray(W, dtype=np.float64)
    dz = np.asarray(dh, dtype=np.float64)[rows]
    if relu:
        dz = dz * (np.asarray(h_out)[rows] > 0)
    dW = np.asarray(agg, dtype=np.float64).T @ dz
    db = dz.sum(axis=0)
    dm = dz @ W.T
    dsrc = np.zeros((n_src, W.shape[0]), dtype=np.float64)
    for k, r in enumerate(rows):
        nb = col[start[r]:end[r]]
        share = dm[k] / float(len(nb) + 1)
        dsrc[r] += share
        if len(nb):
            np.add.at(dsrc, nb, share)
    return dsrc, dW, db


def backward(mb, rec, weights, labels, compute_dtype="f32", model="sage"):
    """loss.backward() of Alg. 1 over the pruned mini-batch of one `iteration` record.

    Gradients flow from the seeds down through the rows that were computed (V_normal); a fetched embedding
    receives its gradient (that is the "zero-cost" signal of Section 4.1.1) and passes nothing below.
    Returns dH[l] (float64 by position, l = 1..L), gnorm[l] = row norms rounded to float32 (l = 1..L-1),
    dW[l], db[l]. The gradient with respect to raw features is not formed.
    In the bf16 setting dH(l) is carried as float32 between the layers (each layer's result rounded once to float32,
    as the device stores it) and the matrix products take bf16 operands (`layer_backward`).
    """
    L = mb.num_layers
    H, AGG, look = rec["H"], rec["AGG"], rec["look"]
    dH = {L: softmax_xent_grad(H[L], labels)}
    dW, db = {}, {}
    for l in range(L, 0, -1):
        rows = look[l]["normal_pos"]
        h_prev = np.asarray(H[l - 1])
        if model == "gcn":
            dsrc, dW[l], db[l] = layer_backward_gcn(mb.start[l], mb.end[l], mb.col[l], rows, dH[l], H[l], AGG[l], weights[l][0],
                                                    len(mb.ids[l - 1]), relu=(l < L))
        else:
            h_self = round_bf16(h_prev[rows].astype(np.float64)) if compute_dtype == "bf16" else h_prev[rows]
            dh_l = dH[l].astype(np.float32) if compute_dtype == "bf16" else dH[l]
            dsrc, dW[l], db[l] = layer_backward(mb.start[l], mb.end[l], mb.col[l], rows, dh_l, H[l], h_self, AGG[l], weights[l][0],
                                                len(mb.ids[l - 1]), relu=(l < L), compute_dtype=compute_dtype)
        if l >= 2:
            dH[l - 1] = dsrc
    gnorm = {l: row_norms(dH[l]).astype(np.float32) for l in range(1, L)}
    return dict(dH=dH, gnorm=gnorm, dW=dW, db=db)


# --------------------------------------------------------------------------- Update(C, V_normal, V, h, i, t_stale, p_grad)

def admission_threshold(g_live, p_grad):
    """Threshold tau such that "g < tau" selects the p_grad fraction with the smallest gradient norms.

    k = floor(p_grad * m) with m the number of live nodes (p_grad taken as the float32 the caller
    passes, the product in float64); tau is the value of rank k (0-based, ascending), +inf when
    k >= m, -inf when k = 0. Ties at tau are not admitted, so the result does not depend on order.
    """
    m = len(g_live)
    k = int(np.floor(np.float64(np.float32(p_grad)) * np.float64(m)))
    if k <= 0:
        return -np.inf, k
    if k >= m:
        return np.inf, k
    return float(np.sort(np.asarray(g_live, dtype=np.float32))[k]), k


SAVING_MAX = 2047   # the estimate of saved accesses saturates here


def access_estimate(start, end, col, hit, below=None):
    """Estimated memory accesses a cached embedding of each node of one layer would save (the quantity the policy "for
    accuracy and performance" of Section 7.4 prioritises by; the text does not define it, this is the reading taken).

    It is the number of rows read to produce the node's embedding in this mini-batch, counted along the pruned blocks
    like a tree: a raw feature row is one read (`below` None: the layer below is the input layer), a node served from
    the cache is one read, a computed node reads what its own row of the layer below and each of its remaining
    neighbours read. Saturates at SAVING_MAX at every layer.
    start, end, col: the layer's block after pruning; hit: per position; below: the estimates of the layer below by
    position. Returns one integer per position of the layer.
    """
    n = len(start)
    out = np.zeros(n, dtype=np.int64)
    for j in range(n):
        if hit[j]:
            out[j] = 1
            continue
        total = 1 if below is None else int(below[j])
        for c in range(int(start[j]), int(end[j])):
            total += 1 if below is None else int(below[col[c]])
        out[j] = min(total, SAVING_MAX)
    return out


def cache_update(cache, i, ids, live, hit, gnorm, p_grad, h, saving=None, budget=None):
    """Update of one layer's cache after iteration i (Sections 4.1.1, 4.1.2, ring of 4.2).

    Population: all live nodes of the layer, computed or fetched (the paper's example compares the
    gradient norm of a fetched node with that of a computed one). With tau from
    `admission_threshold`:
      * a hit whose norm is not below tau is checked out: its mapping entry is invalidated;
      * a hit whose norm is below tau stays as it is (its stamp is not refreshed: it was not recomputed);
      * normal nodes with norm below tau are admitted in ascending position order into the slots
        head, head+1, ... (mod capacity): row copied from h, slot owner and stamp = i written, mapping
        entry set. A recycled slot's previous owner stops hitting because the slot no longer names it.
        At most min(budget, capacity) get in (budget None: capacity). If more are admissible, those with the largest
        `saving` (estimated saved accesses by position, see `access_estimate`; None: all equal) are taken, among equal
        ones the lower positions first; without estimates that is the first `capacity` in position order.
      * the header advances by the number admitted.
    Staleness needs no pass of its own: `HistoricalCache.slot_of` enforces the bound.
    Returns counts (admitted, evicted_by_gradient, overwritten_valid, dropped_overflow) and tau.
    """
    n = len(ids)
    live = np.ones(n, dtype=bool) if live is None else np.asarray(live, dtype=bool)
    hit = np.asarray(hit, dtype=bool)
    g = np.asarray(gnorm, dtype=np.float32)
    tau, _ = admission_threshold(g[live], p_grad)
    admitted = evicted = overwritten = dropped = 0
    for j in range(n):
        if live[j] and hit[j] and not (g[j] < tau):
            cache.map[ids[j]] = -1
            evicted += 1
    head = cache.head
    room = cache.capacity if budget is None else min(int(budget), cache.capacity)
    candidates = [j for j in range(n) if live[j] and not hit[j] and g[j] < tau]
    if len(candidates) > room:
        worth = (lambda j: 0) if saving is None else (lambda j: min(int(saving[j]), SAVING_MAX))
        chosen = set(sorted(candidates, key=lambda j: (-worth(j), j))[:room])
    else:
        chosen = set(candidates)
    for j in candidates:
        if j not in chosen:
            dropped += 1
            continue
        s = (head + admitted) % cache.capacity
        old = int(cache.slot_node[s])
        if old >= 0 and cache.slot_of(old, i + 1) == s:
            overwritten += 1
        cache.slot_node[s] = ids[j]
        cache.slot_stamp[s] = i
        cache.store(s, h[j])
        cache.map[ids[j]] = s
        admitted += 1
    cache.head = (head + admitted) % cache.capacity if cache.capacity else 0
    cache.used = cache.capacity if head + admitted >= cache.capacity else max(cache.used, head + admitted)
    return dict(admitted=admitted, evicted_by_gradient=evicted, overwritten=overwritten, dropped_overflow=dropped, tau=tau)


# --------------------------------------------------------------------------- the whole iteration

def check_minibatch(mb):
    """Structural checks of a sampled mini-batch (layout described in the sampler): raises on violation."""
    L = mb.num_layers
    for l in range(L + 1):
        assert len(np.unique(mb.ids[l])) == len(mb.ids[l]), "node ids repeat within a layer"
    for l in range(1, L + 1):
        n = len(mb.ids[l])
        assert len(mb.start[l]) == n and len(mb.end[l]) == n
        assert np.array_equal(mb.ids[l - 1][:n], mb.ids[l]), "layer l-1 must begin with layer l"
        assert np.all(mb.start[l] <= mb.end[l]) and (n == 0 or mb.end[l].max() <= len(mb.col[l]))
        assert n == 0 or np.all(mb.start[l][1:] >= mb.end[l][:-1])
        if len(mb.col[l]):
            assert mb.col[l].min() >= 0 and mb.col[l].max() < len(mb.ids[l - 1])


def iteration(mb, i, caches, feature_rows, weights, gnorms, p_grad, dims, feat_dtype="f32", compute_dtype="f32",
              update=True, feature_side=None, labels=None, stabilization=0, model="sage", admit_budget=None):
    """One pass of Algorithm 1 without loss/backward (gradient norms are given).

    mb        sampled mini-batch (its `end` arrays are modified: pruning)
    caches    {l: HistoricalCache} for l = 1..L-1 (missing or None: that layer is never looked up)
    feature_rows(ids) -> raw feature rows; weights[l] = (W_l, b_l); gnorms[l] = norms by position
    dims      [d_0..d_L]
    feature_side   optional BidirectionalCache whose rings are `caches`: raw features are loaded through it
    model     "sage": GraphSAGE-mean layers (`aggregate`, `linear`, W_l [2*d, d']); "gcn": GCN layers (`aggregate_gcn`,
              `linear_gcn`, W_l [d, d']), fp32 only
    stabilization   length of the stabilization period (Section 4.1.4): in iterations i < stabilization the historical
              cache is disabled (no lookup, no admission: regular mini-batch training), afterwards it is active
    admit_budget   optional {l: rows}: the access-aware admission policy. A layer's update admits at most that many rows
              and, when more are admissible, prefers those with the largest `access_estimate`
    labels    optional class of every seed: the gradient norms then come from `backward` (softmax cross-entropy on
              H(L)) and `gnorms` is ignored
    Types: H(0) in feat_dtype; H(l), AGG(l) for l >= 1 in compute_dtype except H(L) which is fp32.
    In the bf16 setting the operands of the product are bf16: the own rows, the mean and W are each rounded to bf16
    before it (a no-op for operands stored as bf16); products, sums, bias and ReLU stay in higher precision, and the
    result is rounded once to the layer's storage type.
    Returns a record of every intermediate the GPU path exposes.
    """
    L = mb.num_layers
    rec = dict(layers={})
    cache_active = i >= stabilization
    if not cache_active:
        caches = {}
    live = [None] * (L + 1)
    look = [None] * (L + 1)
    live[L] = np.ones(len(mb.ids[L]), dtype=bool)
    for l in range(L, -1, -1):
        cache = caches.get(l) if (1 <= l <= L - 1) else None
        if l >= 1:
            look[l] = lookup_prune(cache, i, mb.ids[l], live[l], mb.start[l], mb.end[l], mb.col[l], len(mb.ids[l - 1]))
            live[l - 1] = look[l]["live_src"]
        else:
            look[0] = lookup_prune(None, i, mb.ids[0], live[0], None, None, None, 0)
    H = [None] * (L + 1)
    AGG = [None] * (L + 1)
    H[0] = np.zeros((len(mb.ids[0]), dims[0]), dtype=storage_numpy_dtype(feat_dtype))
    input_pos = look[0]["normal_pos"]
    from_buffer = np.zeros(len(input_pos), dtype=bool)
    if feature_side is None:
        gather(feature_rows, mb.ids[0][input_pos], H[0], input_pos)
    elif len(input_pos):
        rows, from_buffer = feature_side.load(mb.ids[0][input_pos], feature_rows)
        H[0][input_pos] = rows
    for l in range(1, L + 1):
        out_dtype = "f32" if l == L else compute_dtype
        H[l] = np.zeros((len(mb.ids[l]), dims[l]), dtype=storage_numpy_dtype(out_dtype))
        if 1 <= l <= L - 1 and caches.get(l) is not None and len(look[l]["hit_pos"]):
            c = caches[l]
            gather(lambda s: c.table[s], look[l]["hit_slot"], H[l], look[l]["hit_pos"])
        rows = look[l]["normal_pos"]
        W, b = weights[l]
        if model == "gcn":
            assert compute_dtype == "f32"
            AGG[l] = round_to(aggregate_gcn(mb.start[l], mb.end[l], mb.col[l], rows, H[l - 1]), "f32")
            H[l][rows] = round_to(linear_gcn(AGG[l], W, b, relu=(l < L)), out_dtype)
            continue
        agg64 = aggregate(mb.start[l], mb.end[l], mb.col[l], rows, H[l - 1])
        if compute_dtype == "bf16":
            AGG[l] = round_bf16(agg64)
            h_self = round_bf16(H[l - 1][rows].astype(np.float64))
            W = round_bf16(W)
        else:
            AGG[l] = round_to(agg64, "f32")
            h_self = H[l - 1][rows]
        z = linear(h_self, AGG[l], W, b, relu=(l < L))
        H[l][rows] = round_to(z, out_dtype)
    stats = {}
    rec.update(live=live, look=look, H=H, AGG=AGG)
    if labels is not None:
        rec["backward"] = backward(mb, rec, weights, labels, compute_dtype, model)
        gnorms = rec["backward"]["gnorm"]
    if not cache_active:
        stats = {l: dict(admitted=0, evicted_by_gradient=0, overwritten=0, dropped_overflow=0, tau=None) for l in range(1, L)}
    saving = {}
    if admit_budget is not None:
        below = None
        for l in range(1, L):
            saving[l] = below = access_estimate(mb.start[l], mb.end[l], mb.col[l], look[l]["hit"], below)
        rec["saving"] = saving
    if update:
        for l in range(1, L):
            if caches.get(l) is not None:
                stats[l] = cache_update(caches[l], i, mb.ids[l], live[l], look[l]["hit"], gnorms[l], p_grad, H[l],
                                        saving=saving.get(l), budget=None if admit_budget is None else admit_budget.get(l))
    rec.update(live=live, look=look, H=H, AGG=AGG, stats=stats, feature_from_buffer=from_buffer)
    return rec
