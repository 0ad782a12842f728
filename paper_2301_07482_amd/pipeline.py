"""One training iteration's data path (Algorithm 1 without loss/backward) as a sequence of C-ABI calls.

This module only owns device buffers (torch tensors) and the order of the calls; every computation is
done by the HIP kernels behind `binding`. Nothing is copied back to the host between calls: element
counts stay in device memory and each call is launched over a static upper bound.
"""
import numpy as np
import torch

from . import binding as B

TORCH_DTYPE = {B.FG_F32: torch.float32, B.FG_F16: torch.float16, B.FG_BF16: torch.bfloat16}
DTYPE_CODE = {"f32": B.FG_F32, "f16": B.FG_F16, "bf16": B.FG_BF16}


def layer_bounds(batch, fanouts, num_nodes):
    """Static upper bounds n_L..n_0 (index l) and nnz_l of a sampled mini-batch."""
    L = len(fanouts)
    n = [0] * (L + 1)
    nnz = [0] * (L + 1)
    n[L] = batch
    for l in range(L, 0, -1):
        nnz[l] = n[l] * fanouts[l - 1]
        n[l - 1] = min(n[l] + nnz[l], num_nodes)
    return n, nnz


class DeviceBatch:
    """A sampled mini-batch resident in device memory (ids, two-row-array blocks, gradient norms)."""

    def __init__(self, mb, gnorms, device="cuda", labels=None, col_ids=False):
        """gnorms: {layer: norms by position} given from outside, or None when `labels` (the seeds' classes) are given and
        the norms come from the backward pass; the blocks' transposes are then uploaded too."""
        L = mb.num_layers
        self.num_layers = L
        self.ready = None      # the uploads below are complete when they return: nothing for `HotPath.run` to wait for
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
        self.n = [len(x) for x in mb.ids]
        self.n_dev = [None] * (L + 1)       # the layer sizes are host integers
        self.ids = [up(x) for x in mb.ids]
        self.start = [None] + [up(mb.start[l]) for l in range(1, L + 1)]
        self.end = [None] + [up(mb.end[l]) for l in range(1, L + 1)]
        self.col = [None] + [up(mb.col[l]) if len(mb.col[l]) else torch.zeros(1, dtype=torch.int32, device=device)
                             for l in range(1, L + 1)]
        self.nnz = [0] + [len(mb.col[l]) for l in range(1, L + 1)]
        self.gnorm = {l: up(np.asarray(g, dtype=np.float32)) for l, g in (gnorms or {}).items()}
        # block 1's columns as node ids (for the loader that takes them directly): the same block, renumbered
        self.col_ids1 = None
        if col_ids and L >= 1:
            self.col_ids1 = up(mb.ids[0][mb.col[1]].astype(np.int32)) if len(mb.col[1]) else torch.zeros(1, dtype=torch.int32, device=device)
        self.labels = None
        if labels is not None:
            from fg_inputs.sampler import transpose_block
            self.labels = up(np.asarray(labels, dtype=np.int32))
            self.t_start, self.t_end, self.t_row = [None] * (L + 1), [None] * (L + 1), [None] * (L + 1)
            for l in range(2, L + 1):       # the input layer needs no gradient
                ts, te, tr = transpose_block(mb.start[l], mb.end[l], mb.col[l], len(mb.ids[l - 1]))
                self.t_start[l], self.t_end[l] = up(ts), up(te)
                self.t_row[l] = up(tr) if len(tr) else torch.zeros(1, dtype=torch.int32, device=device)


class SampledBatch:
    """A mini-batch sampled on the device (`DeviceSampler.sample`): the same fields as `DeviceBatch`; the transposed blocks
    only if the sampler was asked for them, `labels` (the seeds' classes) for the caller to set.

    Until `finish()` the layer sizes exist only in device memory: `n[l]` and `nnz[l]` are the sampler's bounds (the arrays
    hold that many entries; rows at and beyond the count are empty) and `n_dev[l]` is the address of layer l's count, which
    `HotPath.run` hands to the calls that walk whole layers. Nothing then waits for the sampler on the host."""

    def __init__(self, L):
        self.num_layers = L
        self.n, self.nnz = [0] * (L + 1), [0] * (L + 1)
        self.n_dev = [None] * (L + 1)
        self.ids = [None] * (L + 1)
        self.start, self.end, self.col = [None] * (L + 1), [None] * (L + 1), [None] * (L + 1)
        self.col_ids1 = None
        self.gnorm = {}
        self.labels = None
        self.t_start, self.t_end, self.t_row = [None] * (L + 1), [None] * (L + 1), [None] * (L + 1)
        self._counts = self._bound = self._n_seeds = None
        # recorded behind the sampling launches (`DeviceSampler.sample`); a caller that adds to the mini-batch on the device
        # afterwards (norms, labels) records its own event behind that work and puts it here
        self.ready = None

    def finish(self, host_counts=None):
        """Read the layer sizes back (synchronises with the sampling launches) and cut the arrays to them. host_counts: the
        counts already copied to the host by the caller (a pinned copy made on the sampling stream)."""
        L = self.num_layers
        host = (self._counts.cpu() if host_counts is None else host_counts).tolist()   # row l: (nodes of layer l, edges of block l + 1); row L is not written
        host[L][0] = self._n_seeds
        for l in range(L + 1):
            self.n[l] = int(host[l][0])
            self.n_dev[l] = None
            assert self.n[l] <= self._bound[l], "a layer outgrew its bound"
            if l < L:
                self.ids[l] = self.ids[l][:max(self.n[l], 1)]
        for l in range(1, L + 1):
            self.nnz[l] = int(host[l - 1][1])
            self.start[l], self.end[l] = self.start[l][:max(self.n[l], 1)], self.end[l][:max(self.n[l], 1)]
        return self


class DeviceSampler:
    """Samples whole mini-batches with fg_sample_block over an in-neighbour CSR in HBM: one call per block, each layer's
    device-side count feeding the next call. `sample(..., finish=False)` returns at once with the sizes still on the device
    (the path takes them from there); `finish()` reads them back for callers that want host integers."""

    def __init__(self, indptr, indices, num_nodes, fanouts, batch, device="cuda", transposes=False):
        """transposes: also build the transposed blocks of layers 2..L (fg_transpose_block), which the backward pass walks."""
        self.indptr, self.indices = indptr, indices
        self.num_nodes, self.num_edges = int(num_nodes), int(indices.numel())
        self.fanouts = [int(f) for f in fanouts]
        self.L = L = len(self.fanouts)
        self.device = device
        self.bound = [0] * (L + 1)
        self.bound[L] = int(batch)
        for l in range(L, 0, -1):
            self.bound[l - 1] = self.bound[l] * (1 + self.fanouts[l - 1])
        self.out_at, at = {}, 0
        for l in range(L, 0, -1):      # where each output array of a mini-batch starts in its one allocation (256-byte aligned)
            rows, f = self.bound[l], self.fanouts[l - 1]
            offs = []
            tr = transposes and l >= 2      # t_start, t_end over the layer below, t_row over the edges
            for size in (rows, rows, rows * f, self.bound[l - 1], rows * f if l == 1 else 0,
                         self.bound[l - 1] if tr else 0, self.bound[l - 1] if tr else 0, rows * f if tr else 0):
                offs.append(at)
                at += -(-max(size, 1) // 64) * 64
            self.out_at[l] = offs
        self.out_elems = at
        self.ws_bytes = max(B.fg_sample_block_workspace_bytes(self.bound[l], self.fanouts[l - 1]) for l in range(1, L + 1))
        self.transposes = transposes
        if transposes:
            self.ws_bytes = max([self.ws_bytes] + [B.fg_transpose_block_workspace_bytes(self.bound[l - 1]) for l in range(2, L + 1)])
        self.ws = torch.zeros(self.ws_bytes, dtype=torch.uint8, device=device)

    def buffers(self):
        """The output memory of one mini-batch (`sample(..., out=...)`): allocate it ahead of time, or reuse a consumed one."""
        return (torch.empty(self.out_elems, dtype=torch.int32, device=self.device),
                torch.empty((self.L + 1, 2), dtype=torch.int64, device=self.device))

    def sample(self, seeds, key, finish=True, out=None, ready=True):
        """seeds: int32 device tensor of distinct node ids (at most `batch`); key: the mini-batch's 64-bit key.
        finish=False: only the launches; `SampledBatch.finish()` later reads the counts back (sampling ahead of the
        consumer needs no synchronisation per mini-batch that way). ready=False: no event is recorded behind the launches
        (the caller sets the mini-batch's `ready` itself, behind whatever it adds on the device)."""
        L, dev = self.L, self.device
        st = torch.cuda.current_stream().cuda_stream
        bt = SampledBatch(L)
        n_seeds = int(seeds.numel())
        assert n_seeds <= self.bound[L]
        buf, counts = out if out is not None else self.buffers()   # every output array; counts row l: nodes of layer l, edges of block l + 1
        bt.ids[L] = seeds
        cp = counts.data_ptr()
        for l in range(L, 0, -1):
            f = self.fanouts[l - 1]
            rows = self.bound[l] if l < L else n_seeds
            o = self.out_at[l]
            bt.start[l], bt.end[l] = buf[o[0]:o[0] + max(rows, 1)], buf[o[1]:o[1] + max(rows, 1)]
            bt.col[l], bt.ids[l - 1] = buf[o[2]:o[2] + max(rows * f, 1)], buf[o[3]:o[3] + self.bound[l - 1]]
            col_ids = buf[o[4]:o[4] + max(rows * f, 1)] if l == 1 else None
            B.fg_sample_block(self.indptr, self.indices, self.num_nodes, self.num_edges, bt.ids[l], None if l == L else cp + 16 * l,
                              rows, f, int(key), l, bt.start[l], bt.end[l], bt.col[l], col_ids, bt.ids[l - 1], self.bound[l - 1],
                              cp + 16 * (l - 1), self.ws, self.ws_bytes, st)
            if l == 1:
                bt.col_ids1 = col_ids
            if self.transposes and l >= 2:
                nb = self.bound[l - 1]
                bt.t_start[l], bt.t_end[l], bt.t_row[l] = buf[o[5]:o[5] + nb], buf[o[6]:o[6] + nb], buf[o[7]:o[7] + max(rows * f, 1)]
                B.fg_transpose_block(bt.start[l], bt.end[l], bt.col[l], None if l == L else cp + 16 * l, rows, cp + 16 * (l - 1), nb,
                                     rows * f, bt.t_start[l], bt.t_end[l], bt.t_row[l], self.ws, self.ws_bytes, st)
        bt._counts, bt._bound, bt._n_seeds = counts, self.bound, n_seeds
        # until the sizes are read back: the bounds, and where each layer's count lives
        for l in range(L + 1):
            bt.n[l] = self.bound[l] if l < L else n_seeds
            bt.n_dev[l] = cp + 16 * l if l < L else None
        for l in range(1, L + 1):
            bt.nnz[l] = (self.bound[l] if l < L else n_seeds) * self.fanouts[l - 1]
        if ready:
            bt.ready = torch.cuda.Event()
            bt.ready.record(torch.cuda.current_stream())
        return bt.finish() if finish else bt


def _no_tick(name, stream=None):
    return None


class HotPath:
    """Work buffers, cache and weights of one model; `run(batch, it)` executes one iteration."""

    def __init__(self, num_nodes, dims, fanouts, batch, capacity, t_stale, p_grad, features, feat_dtype, compute_dtype,
                 weights, features_on_host=False, device="cuda", use_cache=True, update_all=True, fetch_all=True, fused_input=False,
                 one_launch_top_down=True, log_ring=256, hot_ids=None, buffer_bytes=None, backward=False, weight_grads=False, stabilization=0, model="sage", fuse_small_layers=False,
                 fetch_with_loader=True, admit_budget=None, overlap_update=True, overlap_min_rows=0, copy_own_rows=False):
        self.device = device
        self.L = L = len(fanouts)
        self.dims = list(dims)
        self.num_nodes = num_nodes
        self.p_grad = float(p_grad)
        self.feat = features
        self.feat_code = DTYPE_CODE[feat_dtype]
        self.comp_code = DTYPE_CODE[compute_dtype]
        self.on_host = 1 if features_on_host else 0
        self.use_cache = use_cache
        # fused_input: layer 1 aggregates straight from the feature table (fg_gather_aggregate); only the layer-1
        # nodes' own rows are gathered into H[0] and the top-down pass stops at layer 1
        self.fused_input = fused_input
        # copy_own_rows: the loader also copies the layer-1 nodes' own rows into H[0] for the dense update. Off: the dense
        # update of layer 1 reads them from the table itself by node id (fg_linear_ids), where `own_rows_from_table` allows
        self.copy_own_rows = bool(copy_own_rows)
        # one_launch_top_down: the whole top-down pass as one call (fg_top_down) instead of one fg_lookup_prune call per layer
        self.one_launch_top_down = one_launch_top_down
        self.n_max, self.nnz_max = layer_bounds(batch, fanouts, num_nodes)
        n = self.n_max
        dev = device
        # embeddings by position: H[0] in the feature type, H[l] in the compute type, H[L] fp32
        self.h_code = [self.feat_code] + [self.comp_code] * (L - 1) + [B.FG_F32]
        self.H = [torch.zeros((n[l], dims[l]), dtype=TORCH_DTYPE[self.h_code[l]], device=dev) for l in range(L + 1)]
        self.agg_code = B.FG_F32 if self.comp_code == B.FG_F32 else B.FG_BF16
        agg_elems = max(n[l] * dims[l - 1] for l in range(1, L + 1))
        # the neighbour means of a layer, in list order; with weight gradients every layer keeps its own until the backward pass
        self.weight_grads = bool(weight_grads and backward)
        if self.weight_grads:
            self.AGG_l = [None] + [torch.zeros(n[l] * dims[l - 1], dtype=TORCH_DTYPE[self.agg_code], device=dev) for l in range(1, L + 1)]
        else:
            shared = torch.zeros(agg_elems, dtype=TORCH_DTYPE[self.agg_code], device=dev)
            self.AGG_l = [None] + [shared] * L
        self.AGG = self.AGG_l[L]
        # model "gcn": GCN layers (propagation incl. the node itself, one weight matrix [d_in x d_out]); fp32.
        # The mean's first half goes to a by-position buffer, its second half to AGG in list order (what fg_linear reads).
        self.model = model
        # optional: layers with few rows (the seed layer) run aggregation and dense update as one launch (measured no faster
        # than the two launches, so off by default); not when the weight gradients need the means afterwards
        self.fuse_small_layers = bool(fuse_small_layers) and model == "sage" and self.comp_code == B.FG_F32 and not self.weight_grads
        if model == "gcn":
            assert self.comp_code == B.FG_F32 and self.feat_code == B.FG_F32, "GCN layers: fp32"
            if self.weight_grads:   # like the means: every layer keeps its own until the backward pass
                self.MEANPOS_l = [None] + [torch.zeros(n[l] * (dims[l - 1] // 2), dtype=torch.float32, device=dev) for l in range(1, L + 1)]
            else:
                shared_pos = torch.zeros(max(n[l] * (dims[l - 1] // 2) for l in range(1, L + 1)), dtype=torch.float32, device=dev)
                self.MEANPOS_l = [None] + [shared_pos] * L
            self.MEANPOS = self.MEANPOS_l[L]
        self.live = [torch.zeros(n[l], dtype=torch.uint8, device=dev) for l in range(L + 1)]
        self.hit = [torch.zeros(n[l], dtype=torch.uint8, device=dev) for l in range(L + 1)]
        self.saving = [torch.zeros(n[l] if admit_budget else 0, dtype=torch.int32, device=dev) for l in range(L + 1)]
        self.hit_pos = [torch.zeros(n[l], dtype=torch.int32, device=dev) for l in range(L + 1)]
        self.hit_slot = [torch.zeros(n[l], dtype=torch.int32, device=dev) for l in range(L + 1)]
        self.normal_pos = [torch.zeros(n[l], dtype=torch.int32, device=dev) for l in range(L + 1)]
        self.input_ids = torch.zeros(n[0], dtype=torch.int32, device=dev)
        self.self_ids = torch.zeros(n[1], dtype=torch.int32, device=dev)
        # what the top-down pass writes exists three times (iteration it uses set it % 3), so that the pass for the next
        # mini-batch can run while this one's layers are computed (`run(..., next_bt=...)`) and the previous one's
        # admitted rows are still being copied: the second stream then waits for nothing younger than the row copy of
        # two iterations ago, and its chain selection -> next top-down pass can start before this iteration's loader
        mk = lambda dt: [torch.zeros(n[l], dtype=dt, device=dev) for l in range(L + 1)]
        more = lambda: dict(live=mk(torch.uint8), hit=mk(torch.uint8), hit_pos=mk(torch.int32), hit_slot=mk(torch.int32),
                            normal_pos=mk(torch.int32), input_ids=torch.zeros_like(self.input_ids), self_ids=torch.zeros_like(self.self_ids))
        self._lists = [dict(live=self.live, hit=self.hit, hit_pos=self.hit_pos, hit_slot=self.hit_slot, normal_pos=self.normal_pos,
                            input_ids=self.input_ids, self_ids=self.self_ids), more(), more()]
        self._td_for = None      # (iteration, mini-batch) whose top-down pass has already been launched on the second stream
        self._ready_waited = None  # the mini-batch whose `ready` event the second stream waited for in the previous call
        self._row_copy_due = None  # (iteration, descriptors) of a selection whose rows are not copied yet
        # device-side counts/stats are kept per iteration in a ring, so a timed loop can be read back afterwards
        self.ring = int(log_ring)
        self.counts_log = torch.zeros((self.ring, L + 1, 3), dtype=torch.int64, device=dev)
        self.stats_log = torch.zeros((self.ring, L + 1, 4), dtype=torch.int64, device=dev)
        self.counts = self.counts_log[0]
        self.stats = self.stats_log[0]
        ws_bytes = max(max(B.fg_workspace_bytes(B.FG_WS_LOOKUP_PRUNE, n[l]) for l in range(L + 1)),
                       max([B.fg_workspace_bytes(B.FG_WS_CACHE_UPDATE, n[l]) for l in range(1, L)] or [0]))
        self.ws = torch.zeros(ws_bytes + 256, dtype=torch.uint8, device=dev)
        self.ws_bytes = ws_bytes
        # workspace of fg_top_down: zero-filled once, then kept all-zero by the calls themselves
        self.ws_td_bytes = B.fg_top_down_workspace_bytes(B.top_down_layers([dict(n=n[l]) for l in range(L, -1, -1)]))
        self.ws_td = torch.zeros(self.ws_td_bytes + 256, dtype=torch.uint8, device=dev)
        # all caches are updated by one call after the last layer (the last loop of Algorithm 1)
        self.update_all = update_all
        self.fetch_all = fetch_all   # the cached rows of all layers are fetched by one call right after the top-down pass
        self.fetch_with_loader = fetch_with_loader  # ... or inside the id-column loader's launch, where that loader runs
        # selection part of the update (and the next top-down pass) on a second stream beside the layers (norms given from
        # outside). Below about 65 k input rows per mini-batch the layers are too short to hide anything and the cross-stream
        # waits cost more than they save: callers that time small workloads pass overlap_min_rows.
        overlap_update = overlap_update and self.n_max[0] >= overlap_min_rows
        self.overlap_update = overlap_update
        self.side = torch.cuda.Stream(device=device) if overlap_update else None
        self.ev_pruned, self.ev_selected, self.ev_next_pruned = (torch.cuda.Event() for _ in range(3))
        self.ev_done = [torch.cuda.Event(), torch.cuda.Event()]     # row copy of iteration it: ev_done[it % 2]
        self.ev_bw = [torch.cuda.Event() for _ in range(L + 1)]
        self.admit_budget = dict(admit_budget) if admit_budget else None   # {layer: rows per update}: access-aware admission
        assert not (self.admit_budget and not update_all), "the access-aware admission needs fg_cache_update_all"
        self.ws_upd_bytes = sum(B.fg_workspace_bytes(B.FG_WS_CACHE_UPDATE, n[l]) for l in range(1, L))
        # the update's workspace exists twice (iteration it uses half it % 2): the selection of an iteration writes what
        # that iteration's row copy reads, and the next selection may run before that copy
        self.ws_upd_stride = -(-self.ws_upd_bytes // 256) * 256
        self.ws_upd = torch.zeros(2 * self.ws_upd_stride + 256, dtype=torch.uint8, device=dev)
        self.W = {}
        self.Wt = {}
        self.bias = {}
        wt = TORCH_DTYPE[self.comp_code]
        for l in range(1, L + 1):
            W, b = weights[l]
            self.W[l] = torch.from_numpy(np.ascontiguousarray(W)).to(dev).to(wt).contiguous()
            if self.comp_code == B.FG_BF16:      # the layout the bf16 dense update reads fastest (fg_linear_wt); set up once
                self.Wt[l] = self.W[l].t().contiguous()
            self.bias[l] = torch.from_numpy(np.ascontiguousarray(b)).to(dev)
        # backward: the gradient norms of the update come from the backward pass (softmax cross-entropy on H[L] against
        # the batch's labels) instead of from the batch. Gradients are fp32 in every setting; the bf16 model rounds the
        # operands of the backward matrix products as the forward ones
        self.backward = backward
        self.bw_kind = "gcn" if model == "gcn" else ("sage" if self.comp_code == B.FG_F32 else "bf16")
        if backward:
            assert self.comp_code in (B.FG_F32, B.FG_BF16), "the backward pass is for the fp32 and the bf16 model"
            self.dH = [None] + [torch.zeros((n[l], dims[l]), dtype=torch.float32, device=dev) for l in range(1, L + 1)]
            self.gnorm = [None] + [torch.zeros(max(n[l], 1), dtype=torch.float32, device=dev) for l in range(1, L)]
            self.ws_bw_bytes = max([B.fg_layer_backward_workspace_bytes(n[l], n[l], dims[l - 1], dims[l], kind=self.bw_kind)
                                    for l in range(2, L + 1)] or [0])
            self.ws_bw = torch.zeros(self.ws_bw_bytes + 256, dtype=torch.uint8, device=dev)
            if self.weight_grads:
                assert self.feat_code == B.FG_F32 or self.bw_kind == "bf16", "weight gradients of the fp32 models need fp32 features"
                w_rows = [None] + [(1 if model == "gcn" else 2) * dims[l - 1] for l in range(1, L + 1)]
                self.dW = [None] + [torch.zeros((w_rows[l], dims[l]), dtype=torch.float32, device=dev) for l in range(1, L + 1)]
                self.db = [None] + [torch.zeros(dims[l], dtype=torch.float32, device=dev) for l in range(1, L + 1)]
                wg_bytes = B.fg_layer_backward_weights_bf16_workspace_bytes if self.bw_kind == "bf16" else B.fg_layer_backward_weights_workspace_bytes
                self.ws_wg_bytes = max(wg_bytes(n[l], dims[l - 1], dims[l]) for l in range(1, L + 1))
                self.ws_wg = torch.zeros(self.ws_wg_bytes + 256, dtype=torch.uint8, device=dev)
        self.cache = None
        self.feature_side = False
        if L > 1:
            caps = [capacity] * (L - 1) if np.isscalar(capacity) else list(capacity)
            self.capacity = caps
            cdims = [dims[l] for l in range(1, L)]
            if buffer_bytes is None:
                self.cache = B.fg_cache_create(num_nodes, caps, cdims, self.comp_code, t_stale, self._stream())
            else:
                self.cache = B.fg_cache_create_bidirectional(num_nodes, caps, cdims, self.comp_code, t_stale, buffer_bytes,
                                                             self._stream())
            if stabilization:
                B.fg_cache_set_stabilization(self.cache, int(stabilization))
            # hot_ids (hottest first): their raw features are placed on the feature side of the cache's buffer and the
            # loader reads them from there while no embedding has been written over them
            if hot_ids is not None and len(hot_ids):
                self.hot_ids = torch.from_numpy(np.ascontiguousarray(hot_ids, dtype=np.int32)).to(dev)
                d0b = dims[0] * B.DTYPE_SIZE[self.feat_code]
                B.fg_cache_fill_features(self.cache, self.hot_ids, len(hot_ids), self.feat, num_nodes, d0b, d0b, self._stream())
                self.feature_side = True

    def one_launch(self, l, n_rows):
        """Whether layer l with n_rows positions runs aggregation and dense update as one launch (its means are then never stored)."""
        return self.fuse_small_layers and l >= 2 and B.one_launch_layer(n_rows, self.dims[l - 1], self.dims[l])

    def _stream(self):
        return torch.cuda.current_stream().cuda_stream

    def close(self):
        if self.cache is not None:
            self.flush()
            torch.cuda.synchronize()
            B.fg_cache_destroy(self.cache)
            self.cache = None

    def _estimates(self, bt, st):
        for l in range(1, self.L):
            B.fg_access_estimate(bt.start[l], bt.end[l], bt.col[l], bt.nnz[l], bt.n[l], self.hit[l],
                                 self.saving[l - 1] if l > 1 else None, bt.n[l - 1], self.saving[l], st)

    def _update_specs(self, bt, gnorm):
        esz = B.DTYPE_SIZE
        return B.update_layers([dict(layer=l, n=bt.n[l], ids_dev=bt.ids[l], live_dev=self.live[l], hit_dev=self.hit[l],
                                     gnorm_dev=gnorm[l], h_dev=self.H[l], h_stride=self.dims[l] * esz[self.h_code[l]],
                                     stats_dev=self.stats.data_ptr() + l * 32,
                                     saving_dev=self.saving[l] if self.admit_budget else None,
                                     max_admit=int(self.admit_budget.get(l, 0)) if self.admit_budget else 0, n_dev=bt.n_dev[l])
                                for l in range(1, self.L)])

    def _ws_upd(self, it):
        return self.ws_upd.data_ptr() + (it % 2) * self.ws_upd_stride

    def _cnt(self, l, k):
        return self.counts.data_ptr() + (l * 3 + k) * 8

    def _top_down(self, bt, it, st, tick):
        """Lookup, prune, V_normal for layers L .. 0 (or 1 with the fused loader) of mini-batch `bt` on stream `st`, into the
        currently bound lists."""
        L, fused = self.L, self.fused_input
        lowest = 1 if fused else 0

        def layer_args(l):
            has_block = l >= 1
            want_live_below = has_block and not (fused and l == 1)
            return dict(cache_layer=l if (self.use_cache and self.cache is not None and 1 <= l <= L - 1) else 0,
                        ids_dev=bt.ids[l], n=bt.n[l], live_dev=None if l == L else self.live[l],
                        row_start_dev=bt.start[l] if has_block else None, row_end_dev=bt.end[l] if has_block else None,
                        col_dev=bt.col[l] if has_block else None, nnz=bt.nnz[l] if has_block else 0,
                        n_src=bt.n[l - 1] if has_block else 0, live_src_dev=self.live[l - 1] if want_live_below else None,
                        hit_dev=self.hit[l], hit_pos_dev=self.hit_pos[l], hit_slot_dev=self.hit_slot[l],
                        normal_pos_dev=self.normal_pos[l],
                        normal_ids_dev=self.input_ids if l == 0 else (self.self_ids if (fused and l == 1) else None),
                        counts_dev=self._cnt(l, 0), n_dev=bt.n_dev[l])

        if self.one_launch_top_down:
            tick("top_down")
            layers = B.top_down_layers([layer_args(l) for l in range(L, lowest - 1, -1)])
            B.fg_top_down(self.cache if self.use_cache else None, it, layers, self.ws_td, self.ws_td_bytes, st)
        else:
            for l in range(L, lowest - 1, -1):
                a = layer_args(l)
                tick(f"lookup_prune[{l}]")
                B.fg_lookup_prune(self.cache if a["cache_layer"] else None, l, it, a["ids_dev"], a["n"], a["live_dev"],
                                  a["row_start_dev"], a["row_end_dev"], a["col_dev"], a["nnz"], a["n_src"], a["live_src_dev"],
                                  a["hit_dev"], a["hit_pos_dev"], a["hit_slot_dev"], a["normal_pos_dev"], a["normal_ids_dev"],
                                  a["counts_dev"], self.ws, self.ws_bytes, st)

    def flush(self, selection_done=False, main=None):
        """Copy the rows admitted by the last iteration into the cache, if that is still due (`run` leaves it to the next
        call when that call's top-down pass is already on the second stream). Called by everything that reads the cache."""
        if self._row_copy_due is None:
            return
        it, specs = self._row_copy_due
        self._row_copy_due = None
        if main is None:
            main = torch.cuda.current_stream()
        if not selection_done:
            main.wait_event(self.ev_selected)
        B.fg_cache_update_commit(self.cache, it, specs, self._ws_upd(it), self.ws_upd_bytes, main.cuda_stream)
        self.ev_done[it % 2].record(main)

    def _bind(self, it):
        """Point the per-iteration state (lists of the top-down pass, counters, statistics) at iteration `it`'s copies."""
        self.__dict__.update(self._lists[it % 3])
        self.counts = self.counts_log[it % self.ring]
        self.stats = self.stats_log[it % self.ring]

    def run(self, bt, it, update=True, timer=None, next_bt=None, hold_second_stream=False):
        """One iteration on torch's current stream. `timer(name, stream)` (optional) is called before each C-ABI call
        and with name None after the last call of a stream (stream None = the current stream).
        next_bt: the mini-batch of iteration it + 1, if the caller has it: where the update's selection runs on the second
        stream (see below), the top-down pass of that mini-batch follows it there, beside this iteration's layers, and
        the next call (which must be for that mini-batch and iteration) finds it done.
        hold_second_stream: what this call puts on the second stream starts only when layer 1 is done, so that the loader and
        the layer-1 dense update have the chip to themselves (for a caller that times these two launches).
        Ordering of the inputs: the arrays of `bt` and `next_bt` (norms and labels included) are read on torch's current
        stream and, where the update's selection and the next top-down pass run there, on the second stream, which does not
        follow the current stream call by call (it runs up to an iteration ahead). Arrays that are complete when `run` is
        called need nothing (`DeviceBatch`); a mini-batch still being written on the device carries an event recorded behind
        its last write in `ready` (`DeviceSampler.sample` sets it), and both streams are ordered behind it here (the
        current stream directly when this call runs the top-down pass itself, else through the second stream, which waited
        for it in the call that announced the mini-batch)."""
        L = self.L
        self._bind(it)
        tick = timer if timer is not None else _no_tick
        esz = B.DTYPE_SIZE
        main = torch.cuda.current_stream()      # asked for once: the query costs several microseconds of host time
        st = main.cuda_stream
        do_update = update and self.use_cache and self.cache is not None
        # sizes still on the device: the host integers are bounds, and a layer cannot outgrow the node count
        assert all(bt.n[l] <= self.n_max[l] or bt.n_dev[l] is not None for l in range(L + 1)), "mini-batch larger than the static bounds"
        assert all(d is None for d in bt.n_dev) or (self.one_launch_top_down and (self.update_all or not self.use_cache)), \
            "layer sizes in device memory go through fg_top_down and fg_cache_update_all"
        if any(bt.n[l] > self.n_max[l] for l in range(L + 1)):
            bt.n = [min(bt.n[l], self.n_max[l]) for l in range(L + 1)]
        fused = self.fused_input
        promised = self._td_for is not None
        pruned_ahead = promised and self._td_for[0] == it and self._td_for[1] is bt
        self._td_for = None
        if not pruned_ahead and getattr(bt, "ready", None) is not None:
            main.wait_event(bt.ready)      # this call's own launches are the first to read the mini-batch
        if promised:      # (also when the promise was not kept: that pass writes the lists this call is about to use)
            main.wait_event(self.ev_next_pruned)   # behind the previous selection on that stream
        self.flush(selection_done=promised, main=main)
        if not pruned_ahead:
            self._top_down(bt, it, st, tick)

        cached_layers = list(range(1, L)) if (self.use_cache and self.cache is not None) else []
        # With gradient norms given from outside nothing of the update but its row copy depends on the layers computed below:
        # threshold, check-outs, admissions and slots are decided now, on a second stream, beside the loader and the layers.
        # (Not with raw features in the cache's buffer: the loader reads the rings' written extents, which the selection
        # advances. Copying the admitted rows over there too, beside the seed layer, measured slower than on this stream.)
        early_select = None

        def second_stream():
            # (every call below names the second stream itself: torch's current stream stays the caller's)
            side, side_st = self.side, self.side.cuda_stream
            for b in (bt, next_bt):      # mini-batches still being written on the device when this call was made
                if b is not None and b is not self._ready_waited and getattr(b, "ready", None) is not None:
                    side.wait_event(b.ready)
            self._ready_waited = next_bt      # (the next call's `bt`: already waited for)
            if not pruned_ahead or hold_second_stream:
                self.ev_pruned.record(main)
                side.wait_event(self.ev_pruned)
            # What this selection and the top-down pass behind it overwrite (half it % 2 of the workspace, set (it + 1) % 3
            # of the lists) was last read by iteration it - 2 and its row copy, which recorded this event (the copy of
            # iteration it - 1, just queued, recorded the other one).
            side.wait_event(self.ev_done[it % 2])
            if self.admit_budget:
                self._estimates(bt, side_st)
            specs = self._update_specs(bt, bt.gnorm)
            B.fg_cache_update_select(self.cache, it, self.p_grad, specs, self._ws_upd(it), self.ws_upd_bytes, side_st)
            self.ev_selected.record(side)
            if next_bt is not None and self.one_launch_top_down:
                # the cache's index is final for this iteration: the next mini-batch can be looked up and pruned now,
                # into the next set of lists (free since the row copy of two iterations ago: ev_done above)
                self._bind(it + 1)
                self._top_down(next_bt, it + 1, side_st, _no_tick)
                self.ev_next_pruned.record(side)
                self._td_for = (it + 1, next_bt)
                self._bind(it)
            return specs

        beside = do_update and self.update_all and self.overlap_update and not self.backward and bool(cached_layers) and not self.feature_side
        held = {"due": False, "specs": None}
        if beside and not hold_second_stream:
            early_select = second_stream()
        elif beside:
            # released at the first call of layer 2, right behind the caller's timer: an event the timer records there closes
            # the span of layer 1's dense update before the release's own event is queued
            timer_tick = tick

            def tick(name, stream=None):
                timer_tick(name, stream)
                if held["due"]:
                    held["due"] = False
                    held["specs"] = second_stream()
        fetch_specs = None
        if self.fetch_all and cached_layers:
            fetch_specs = B.fetch_layers([dict(layer=l, hit_slot_dev=self.hit_slot[l], hit_pos_dev=self.hit_pos[l],
                                               n_hit_dev=self._cnt(l, 1), max_hits=bt.n[l], h_dev=self.H[l], h_rows=bt.n[l],
                                               h_stride=self.dims[l] * esz[self.h_code[l]]) for l in cached_layers])
            # the id-column loader takes the fetch along in its own launch
            rides = (self.fetch_with_loader and fused and self.model == "sage" and not self.feature_side
                     and getattr(bt, "col_ids1", None) is not None and not self.one_launch(1, bt.n[1]))
            if not rides:
                tick("cache_fetch_all")
                B.fg_cache_fetch_all(self.cache, fetch_specs, st)
                fetch_specs = None
        # ---- loader: raw features of the surviving input nodes (fused: done by fg_gather_aggregate below, which also
        #      copies the layer-1 nodes' own rows into H[0])
        d0b = self.dims[0] * esz[self.feat_code]
        if not fused:
            tick("gather_features")
            if self.feature_side:
                B.fg_gather_features(self.cache, self.feat, self.num_nodes, d0b, d0b, self.input_ids, self.normal_pos[0],
                                     self._cnt(0, 2), bt.n[0], self.H[0], bt.n[0], d0b, self.on_host, st)
            else:
                B.fg_gather(self.feat, self.num_nodes, d0b, d0b, self.input_ids, self.normal_pos[0], self._cnt(0, 2), bt.n[0],
                            self.H[0], bt.n[0], d0b, self.on_host, st)
        # ---- bottom-up: cached rows, mean aggregation, dense update
        for l in range(1, L + 1):
            if beside and hold_second_stream and l == 2:     # (a cache has layers, so L >= 2 here)
                held["due"] = True
            in_code, out_code = self.h_code[l - 1], self.h_code[l]
            in_b = self.dims[l - 1] * esz[in_code]
            out_b = self.dims[l] * esz[out_code]
            if l in cached_layers and not self.fetch_all:
                tick(f"cache_fetch[{l}]")
                B.fg_gather(B.fg_cache_table(self.cache, l), self.capacity[l - 1], out_b, out_b, self.hit_slot[l],
                            self.hit_pos[l], self._cnt(l, 1), bt.n[l], self.H[l], bt.n[l], out_b, B.FG_TABLE_HBM_REUSED, st)
            agg_b = self.dims[l - 1] * esz[self.agg_code]
            if self.model == "gcn":
                half = self.dims[l - 1] // 2
                if fused and l == 1:
                    tick("gather_aggregate[1]")
                    B.fg_gather_aggregate_gcn(bt.start[1], bt.end[1], bt.col[1], bt.nnz[1], bt.n[1], self.normal_pos[1],
                                              self._cnt(1, 2), bt.n[1], bt.ids[0], bt.n[0], self.feat, self.num_nodes, d0b,
                                              self.dims[0], self.MEANPOS_l[1], self.AGG_l[1], st)
                else:
                    tick(f"aggregate[{l}]")
                    B.fg_aggregate_gcn(bt.start[l], bt.end[l], bt.col[l], bt.nnz[l], bt.n[l], self.normal_pos[l], self._cnt(l, 2),
                                       bt.n[l], self.H[l - 1], bt.n[l - 1], in_b, self.dims[l - 1], self.MEANPOS_l[l], self.AGG_l[l], st)
                tick(f"linear[{l}]")
                B.fg_linear(self.MEANPOS_l[l], bt.n[l], half * 4, B.FG_F32, self.AGG_l[l], half * 4, self.normal_pos[l], self._cnt(l, 2),
                            bt.n[l], half, self.dims[l], self.W[l], B.FG_F32, self.bias[l], 1 if l < L else 0, self.H[l], bt.n[l],
                            out_b, out_code, st)
                continue
            if self.one_launch(l, bt.n[l]):
                tick(f"aggregate_linear[{l}]")
                B.fg_aggregate_linear(bt.start[l], bt.end[l], bt.col[l], bt.nnz[l], bt.n[l], self.normal_pos[l], self._cnt(l, 2),
                                      bt.n[l], self.H[l - 1], bt.n[l - 1], in_b, self.dims[l - 1], self.dims[l], self.W[l],
                                      self.bias[l], 1 if l < L else 0, None, agg_b, self.H[l], bt.n[l], out_b, st)
                continue
            if fused and l == 1:
                tick("gather_aggregate[1]")
                args = (bt.start[1], bt.end[1], bt.col[1], bt.nnz[1], bt.n[1], self.normal_pos[1], self._cnt(1, 2), bt.n[1],
                        bt.ids[0], bt.n[0], self.feat, self.num_nodes, d0b, self.dims[0], in_code, self.AGG_l[1], agg_b,
                        self.agg_code, self.H[0], d0b, bt.n[0], st)
                if self.feature_side:
                    B.fg_gather_aggregate_features(self.cache, *args)
                elif getattr(bt, "col_ids1", None) is not None:
                    B.fg_gather_aggregate_ids(bt.start[1], bt.end[1], bt.col_ids1, bt.nnz[1], bt.n[1], self.normal_pos[1],
                                              self._cnt(1, 2), bt.n[1], bt.ids[1], self.feat, self.num_nodes, d0b, self.dims[0],
                                              in_code, self.AGG_l[1], agg_b, self.agg_code,
                                              None if self.own_rows_from_table(bt) else self.H[0], d0b, bt.n[0],
                                              self.cache if fetch_specs is not None else None, fetch_specs, st)
                else:
                    B.fg_gather_aggregate(*args)
            else:
                tick(f"aggregate[{l}]")
                B.fg_aggregate(bt.start[l], bt.end[l], bt.col[l], bt.nnz[l], bt.n[l], self.normal_pos[l], self._cnt(l, 2),
                               bt.n[l], self.H[l - 1], bt.n[l - 1], in_b, self.dims[l - 1], in_code, self.AGG_l[l], agg_b,
                               self.agg_code, st)
            tick(f"linear[{l}]")
            if l == 1 and fused and self.own_rows_from_table(bt):
                B.fg_linear_ids(self.feat, self.num_nodes, in_b, in_code, bt.ids[1], self.AGG_l[1], agg_b, self.normal_pos[1],
                                self._cnt(1, 2), bt.n[1], self.dims[0], self.dims[1], self.W[1], self.comp_code, self.bias[1],
                                1 if L > 1 else 0, self.H[1], bt.n[1], out_b, out_code, st)
                continue
            dense, weights = (B.fg_linear_wt, self.Wt[l]) if l in self.Wt else (B.fg_linear, self.W[l])
            dense(self.H[l - 1], bt.n[l - 1], in_b, in_code, self.AGG_l[l], agg_b, self.normal_pos[l], self._cnt(l, 2),
                  bt.n[l], self.dims[l - 1], self.dims[l], weights, self.comp_code, self.bias[l],
                  1 if l < L else 0, self.H[l], bt.n[l], out_b, out_code, st)
        # ---- loss and backward pass down to layer 1: the gradient norms the update admits and checks out by
        gnorm = bt.gnorm
        if self.backward:
            def weight_grads(l, stream):
                act = self.H[l] if l < L else None
                tail = (bt.n[l], self.normal_pos[l], self._cnt(l, 2), bt.n[l])
                if self.bw_kind == "gcn":    # the layer's input rows are the propagated rows: by-position half ‖ list-order half
                    half = self.dims[l - 1] // 2
                    B.fg_layer_backward_weights(self.MEANPOS_l[l], bt.n[l], half * 4, self.AGG_l[l], half * 4, self.dH[l],
                                                self.dims[l] * 4, act, self.dims[l] * 4, *tail, half, self.dims[l],
                                                self.dW[l], self.db[l], self.ws_wg, self.ws_wg_bytes, stream)
                elif self.bw_kind == "bf16":
                    B.fg_layer_backward_weights_bf16(self.H[l - 1], bt.n[l - 1], self.dims[l - 1] * esz[self.h_code[l - 1]],
                                                     self.h_code[l - 1], self.AGG_l[l], self.dims[l - 1] * 2, self.dH[l],
                                                     self.dims[l] * 4, act, self.dims[l] * 2, *tail, self.dims[l - 1],
                                                     self.dims[l], self.dW[l], self.db[l], self.ws_wg, self.ws_wg_bytes, stream)
                else:
                    B.fg_layer_backward_weights(self.H[l - 1], bt.n[l - 1], self.dims[l - 1] * 4, self.AGG_l[l],
                                                self.dims[l - 1] * 4, self.dH[l], self.dims[l] * 4, act, self.dims[l] * 4,
                                                *tail, self.dims[l - 1], self.dims[l], self.dW[l], self.db[l], self.ws_wg,
                                                self.ws_wg_bytes, stream)

            # The weight gradients of a layer need that layer's output gradient and nothing later: with a second stream they
            # run there, each as soon as its dH exists, beside the rest of the backward chain and the cache update.
            wg_beside = self.weight_grads and self.overlap_update and timer is None

            def weight_grads_beside(l):
                self.ev_bw[l].record(torch.cuda.current_stream())
                with torch.cuda.stream(self.side):
                    self.side.wait_event(self.ev_bw[l])
                    weight_grads(l, self.side.cuda_stream)

            tick("loss_grad")
            B.fg_softmax_xent_grad(self.H[L], self.dims[L] * 4, bt.labels, bt.n[L], self.dims[L], self.dH[L], self.dims[L] * 4, st)
            if wg_beside:
                weight_grads_beside(L)
            for l in range(L, 1, -1):
                tick(f"layer_backward[{l}]")
                B.fg_layer_backward(self.dH[l], self.dims[l] * 4, self.H[l] if l < L else None, self.dims[l] * esz[self.h_code[l]],
                                    bt.n[l], self.normal_pos[l], self._cnt(l, 2), bt.n[l], self.live[l] if l < L else None,
                                    self.hit[l], bt.start[l], bt.end[l], bt.t_start[l], bt.t_end[l], bt.t_row[l], bt.nnz[l],
                                    bt.n[l - 1], self.dims[l - 1], self.dims[l], self.W[l], self.dH[l - 1], self.dims[l - 1] * 4,
                                    self.gnorm[l - 1], self.ws_bw, self.ws_bw_bytes, st, kind=self.bw_kind)   # with the row norms of dH[l-1]
                if wg_beside:
                    weight_grads_beside(l - 1)
            gnorm = self.gnorm
            if self.weight_grads and not wg_beside:
                for l in range(L, 0, -1):
                    tick(f"weight_grads[{l}]")
                    weight_grads(l, st)
        # ---- update of the caches
        if held["due"]:           # no timed call came after layer 1
            held["due"] = False
            held["specs"] = second_stream()
        if held["specs"] is not None:
            early_select = held["specs"]
        if early_select is not None:      # the selection ran beside the layers: only the admitted rows are left to copy
            self._row_copy_due = (it, early_select)
            if self._td_for is None:      # otherwise the next call does it, behind the wait it has anyway (one wait less per step)
                tick("cache_update_commit")
                self.flush()
        elif do_update and self.update_all:
            if self.admit_budget:   # access-aware admission: the estimates, bottom-up over the pruned blocks
                tick("access_estimate")
                self._estimates(bt, st)
            tick("cache_update_all")
            B.fg_cache_update_all(self.cache, it, self.p_grad, self._update_specs(bt, gnorm), self._ws_upd(it), self.ws_upd_bytes, st)
        elif do_update:
            for l in range(1, L):
                out_b = self.dims[l] * esz[self.h_code[l]]
                tick(f"cache_update[{l}]")
                B.fg_cache_update(self.cache, l, it, bt.ids[l], bt.n[l], self.live[l], self.hit[l], gnorm[l],
                                  self.p_grad, self.H[l], out_b, self.stats.data_ptr() + l * 32, self.ws, self.ws_bytes, st)
        if self.backward and self.weight_grads and self.overlap_update and timer is None:
            self.ev_bw[0].record(self.side)       # the next iteration overwrites what the weight gradients read
            torch.cuda.current_stream().wait_event(self.ev_bw[0])
        tick(None)

    def holds_second_stream(self):
        """Whether `run(..., hold_second_stream=True)` has work on a second stream to hold back."""
        return bool(self.overlap_update and self.update_all and self.use_cache and self.cache is not None and self.L > 1
                    and not self.backward and not self.feature_side)

    def own_rows_from_table(self, bt):
        """Whether layer 1's dense update of this mini-batch reads the nodes' own features from the table itself (fp32 table
        in HBM, id-column loader) instead of from a copy the loader makes."""
        return (not self.copy_own_rows and self.fused_input and self.model == "sage" and not self.feature_side and not self.on_host
                and self.comp_code == B.FG_F32 and self.feat_code == B.FG_F32 and not self.weight_grads
                and getattr(bt, "col_ids1", None) is not None and not self.one_launch(1, bt.n[1]))

    # ---- read-back helpers for tests and reports (synchronising) -------------------------------------------
    def snapshot(self, bt):
        """Host copies of what one `run` produced (lists cut to their device-side counts)."""
        self.flush()
        L = self.L
        torch.cuda.synchronize()
        counts = self.counts.cpu().numpy()
        out = dict(counts=counts, stats=self.stats.cpu().numpy(), layers={})
        for l in range(1 if self.fused_input else 0, L + 1):
            n = bt.n[l]
            n_hit, n_norm = int(counts[l, 1]), int(counts[l, 2])
            out["layers"][l] = dict(
                live=(self.live[l][:n].cpu().numpy().astype(bool) if l < L else np.ones(n, dtype=bool)),
                hit=self.hit[l][:n].cpu().numpy().astype(bool),
                hit_pos=self.hit_pos[l][:n_hit].cpu().numpy(), hit_slot=self.hit_slot[l][:n_hit].cpu().numpy(),
                normal_pos=self.normal_pos[l][:n_norm].cpu().numpy(),
                end=None if l == 0 else bt.end[l].cpu().numpy())
        if not self.fused_input:
            out["input_ids"] = self.input_ids[:int(counts[0, 2])].cpu().numpy()
        return out

    def feature_ranks(self, ids_dev, n):
        """Rank on the feature side of each of the first n node ids (device int32), -1 where the row is not (or no longer) there."""
        out = torch.full((max(n, 1),), -7, dtype=torch.int32, device=self.device)
        found = torch.zeros(1, dtype=torch.int64, device=self.device)
        B.fg_feature_lookup(self.cache, ids_dev, None, n, out, found, self._stream())
        torch.cuda.synchronize()
        return out[:n].cpu().numpy(), int(found.item())

    def export_cache(self, layer, it):
        self.flush()
        cap = self.capacity[layer - 1]
        dev = self.device
        nodes = torch.zeros(cap, dtype=torch.int32, device=dev)
        slots = torch.zeros(cap, dtype=torch.int32, device=dev)
        stamps = torch.zeros(cap, dtype=torch.int32, device=dev)
        cnt = torch.zeros(2, dtype=torch.int64, device=dev)
        wsb = B.fg_workspace_bytes(B.FG_WS_EXPORT, cap)
        ws = torch.zeros(wsb, dtype=torch.uint8, device=dev)
        B.fg_cache_export(self.cache, layer, it, nodes, slots, stamps, cnt.data_ptr(), cnt.data_ptr() + 8, ws, wsb,
                          self._stream())
        torch.cuda.synchronize()
        c = int(cnt[0].item())
        return dict(nodes=nodes[:c].cpu().numpy(), slots=slots[:c].cpu().numpy(), stamps=stamps[:c].cpu().numpy(),
                    head=int(cnt[1].item()))

    def cache_rows(self, layer, slots):
        """Rows of the cache table at the given slots, as a host array (bf16 widened to fp32)."""
        self.flush()
        cap, d = self.capacity[layer - 1], self.dims[layer]
        nbytes = cap * d * B.DTYPE_SIZE[self.comp_code]
        tab = _tensor_from_ptr(B.fg_cache_table(self.cache, layer), (cap, d), TORCH_DTYPE[self.comp_code], nbytes, self.device)
        idx = torch.as_tensor(np.asarray(slots, dtype=np.int64), device=self.device)
        return tab[idx].float().cpu().numpy()


# ---- set-up shared by the tests and bench.py (workload -> HotPath); no arithmetic of the method

def make_hotpath(w, feat_table=None, use_cache=True, capacity=None, t_stale=None, p_grad=None, fused_input=False, one_launch_top_down=True, update_all=True, log_ring=256, copy_own_rows=False,
                 hot_ids=None, buffer_bytes=None, backward=False, weight_grads=False, stabilization=0, model="sage",
                 fetch_with_loader=True, admit_budget=None, overlap_update=True, overlap_min_rows=0, fuse_small_layers=False):
    """HotPath for workload `w` with its feature table resident where the workload says."""
    from fg_inputs import device as fdev, workload as wl
    dims = wl.layer_dims(w)
    weights = {l: wl.layer_weights(w, l) for l in range(1, w.num_layers + 1)}
    if model == "gcn":      # one weight matrix per layer: the first d_in rows of the generated pair of panels
        weights = {l: (np.ascontiguousarray(W[:dims[l - 1]]), b) for l, (W, b) in weights.items()}
    if feat_table is None:
        feat_table = fdev.feature_table(w.seed, w.num_nodes, w.feat_dim, w.feat_dtype, w.feat_location)
    hp = HotPath(w.num_nodes, dims, w.fanouts, w.batch, w.cache_capacity if capacity is None else capacity,
                 w.t_stale if t_stale is None else t_stale, w.p_grad if p_grad is None else p_grad, feat_table,
                 w.feat_dtype, w.compute_dtype, weights, features_on_host=(w.feat_location == "host"),
                 use_cache=use_cache, fused_input=fused_input, one_launch_top_down=one_launch_top_down, update_all=update_all,
                 fetch_all=update_all, log_ring=log_ring, hot_ids=hot_ids, buffer_bytes=buffer_bytes, backward=backward, weight_grads=weight_grads, stabilization=stabilization, model=model,
                 fetch_with_loader=fetch_with_loader, admit_budget=admit_budget, overlap_update=overlap_update,
                 overlap_min_rows=overlap_min_rows, fuse_small_layers=fuse_small_layers, copy_own_rows=copy_own_rows)
    return hp, weights, feat_table



def rings_bytes(w, capacity=None):
    """Bytes the rings of workload `w` take at the left end of a shared buffer (each ring starts at a multiple of 256)."""
    from fg_inputs import workload as wl
    dims, es = wl.layer_dims(w), 4 if w.compute_dtype == "f32" else 2
    at = 0
    for l in range(1, w.num_layers):
        at = -(-at // 256) * 256 + (w.cache_capacity if capacity is None else capacity) * dims[l] * es
    return at



class _Ext:
    """Minimal __cuda_array_interface__ holder so torch can view library-owned device memory."""

    def __init__(self, ptr, nbytes):
        self.__cuda_array_interface__ = dict(shape=(nbytes,), typestr="|u1", data=(ptr, False), version=2)


def _tensor_from_ptr(ptr, shape, dtype, nbytes, device):
    raw = torch.as_tensor(_Ext(ptr, nbytes), device=device)
    return raw.view(dtype).view(shape)
