#!/usr/bin/env python3
"""Throughput of the whole hot path (lookup+prune, gather, cache fetch, aggregate, linear, cache update) on one MI355X.

A step is one pass over one sampled mini-batch of the named workload; mini-batches, gradient norms and the
feature table are resident in HBM before the timed region starts. Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large_hbm] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X published dense fp32 matrix rate
BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
PCIE5_X16_GBS = 64.0            # PCIe Gen5 x16, one direction (workloads whose feature table stays in host memory)
PAPER_T_STALE, PAPER_P_GRAD = 200, 0.9   # the paper's default thresholds (Section 7.1)


def _sample_one(args):
    name, it = args
    from fg_inputs import workload as wl
    w = wl.WORKLOADS[name]
    g = wl.make_graph(w)
    mb = wl.minibatch(w, g, it)
    gn = {l: wl.grad_norms(w, it, l, mb.ids[l]) for l in range(1, w.num_layers)}
    return mb, gn, wl.node_labels(w, mb.ids[w.num_layers])


def sample_batches(name, count, workers):
    """Sample `count` mini-batches on host cores (before the GPU is touched: the pool forks)."""
    from concurrent.futures import ProcessPoolExecutor
    jobs = [(name, it) for it in range(count)]
    if workers <= 1:
        return [_sample_one(j) for j in jobs]
    with ProcessPoolExecutor(max_workers=workers) as ex:
        return list(ex.map(_sample_one, jobs, chunksize=1))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="large_hbm")
    ap.add_argument("--scale", type=int, default=1, help="divide node/edge/cache counts (debugging on small boxes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cache", action="store_true", help="run with the historical cache disabled (plain neighbour sampling)")
    ap.add_argument("--no-fuse", action="store_true",
                    help="materialise every input row with fg_gather and aggregate layer 1 from H0 (separate calls) instead "
                         "of aggregating layer 1 straight from the feature table (fg_gather_aggregate)")
    ap.add_argument("--sample-workers", type=int, default=8)
    ap.add_argument("--t-stale", type=int, default=None, help="override the workload's staleness bound (not the headline configuration)")
    ap.add_argument("--p-grad", type=float, default=None, help="override the workload's admission fraction (not the headline configuration)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="fg_set_tuning(KEY, VALUE) before the run (launch-shape experiments; results do not depend on it)")
    ap.add_argument("--per-layer-update", action="store_true",
                    help="one fg_cache_update per layer instead of one fg_cache_update_all")
    ap.add_argument("--bracket-every", type=int, default=10,
                    help="time the two longest calls with HIP events on every k-th step of the timed region")
    ap.add_argument("--feature-rows", type=int, default=0,
                    help="bidirectional cache: place the raw features of this many hottest nodes on the feature side of the "
                         "caches' buffer (beyond the rings, so none is displaced) and load through it")
    ap.add_argument("--backward", action="store_true",
                    help="take the gradient norms of the cache update from the backward pass (softmax cross-entropy on the seeds' "
                         "synthetic labels, layer backward down to layer 1, row norms) instead of the synthetic norms")
    ap.add_argument("--two-launch-seed-layer", action="store_true",
                    help="run the seed layer as fg_aggregate + fg_linear instead of through fg_aggregate_linear (one launch, the "
                         "default where the layer's shape allows it: the two measure the same, the one launch needs no buffer "
                         "for the means)")
    ap.add_argument("--copy-own-rows", action="store_true",
                    help="let the loader copy the layer-1 nodes' own feature rows out for the dense update (fg_linear) instead of "
                         "that update reading them from the table by node id (fg_linear_ids, the default for an fp32 table in HBM)")
    ap.add_argument("--block-positions", action="store_true",
                    help="give the fused loader block 1 with positions as columns (fg_gather_aggregate) instead of node ids "
                         "(fg_gather_aggregate_ids)")
    ap.add_argument("--cache-slots", type=int, default=None, help="override the workload's slots per cached layer (not the headline configuration)")
    ap.add_argument("--access-aware", action="store_true",
                    help="access-aware admission: every update admits at most capacity / t_stale rows per layer, those with "
                         "the largest estimate of saved row reads first (fg_access_estimate, fg_cache_update_all)")
    ap.add_argument("--admit-budget", default=None, metavar="ROWS[,ROWS...]",
                    help="access-aware admission with these budgets for layers 1, 2, ... instead of capacity / t_stale")
    ap.add_argument("--device-sampler", action="store_true",
                    help="sample the mini-batches on the device (fg_sample_block over the graph written out as a CSR in HBM) "
                         "instead of on host cores; the sampling rate is reported under `sampler`, `value` stays the path's rate "
                         "on resident mini-batches")
    ap.add_argument("--no-lookahead", action="store_true",
                    help="do not hand the next mini-batch to the step before it (its top-down pass then runs at the start of its own "
                         "step instead of on the second stream beside the previous step's layers)")
    ap.add_argument("--no-overlap-update", action="store_true",
                    help="run the whole cache update after the last layer on the one stream, instead of its selection part on a "
                         "second stream beside the layers (possible because the gradient norms are given from outside)")
    ap.add_argument("--separate-fetch", action="store_true",
                    help="fetch the cached embeddings with a launch of their own (fg_cache_fetch_all) instead of inside the "
                         "id-column loader's launch")
    ap.add_argument("--model", default="sage", choices=["sage", "gcn"],
                    help="layer type: GraphSAGE-mean (the headline) or GCN (propagation incl. the node itself, one weight matrix)")
    ap.add_argument("--weight-grads", action="store_true",
                    help="with --backward: also form dL/dW and dL/db of every layer (fg_layer_backward_weights)")
    ap.add_argument("--no-policy-paper", action="store_true",
                    help="skip the second measurement with the paper's default thresholds (t_stale 200, p_grad 0.9), reported "
                         "as `policy_paper`")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy before the warm-up, as the known-size "
                         "reference for scaling hardware traffic counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path has no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    from fg_inputs import workload as wl
    w = wl.WORKLOADS[args.workload]
    if args.scale > 1:
        w = w.scaled(args.scale)
        wl.WORKLOADS[w.name] = w
    if args.t_stale is not None or args.p_grad is not None or args.cache_slots is not None:
        import dataclasses
        w = dataclasses.replace(w, name=w.name + "/policy", t_stale=w.t_stale if args.t_stale is None else args.t_stale,
                                p_grad=w.p_grad if args.p_grad is None else args.p_grad,
                                cache_capacity=w.cache_capacity if args.cache_slots is None else args.cache_slots)
        wl.WORKLOADS[w.name] = w
    admit_budget = None
    if args.admit_budget:
        admit_budget = {l + 1: int(v) for l, v in enumerate(args.admit_budget.split(","))}
    elif args.access_aware:      # what a ring of this size can hold for a whole staleness window
        admit_budget = {l: max(1, -(-w.cache_capacity // max(w.t_stale, 1))) for l in range(1, w.num_layers)}
    # The cache reaches its steady state after t_stale + 1 updates (entries admitted by the first update have then aged
    # out): whatever --warmup says, that many untimed iterations run before the timed region; those beyond --warmup are
    # reported as `prefill_steps`.
    prefill = 0 if args.no_cache else max(0, w.t_stale + 1 - args.warmup)
    first_timed = prefill + args.warmup
    total = first_timed + args.steps
    extra = min(args.steps, 20)        # further mini-batches for the per-call breakdown pass after the timed region
    policy_w = None
    if not (args.no_policy_paper or args.no_cache or w.num_layers < 2 or args.backward or args.device_sampler or args.feature_rows
            or args.t_stale is not None or args.p_grad is not None):
        import dataclasses
        policy_w = dataclasses.replace(w, name=w.name + "/paper_policy", t_stale=PAPER_T_STALE, p_grad=PAPER_P_GRAD)
        wl.WORKLOADS[policy_w.name] = policy_w
    n_sampled = total + extra
    if policy_w is not None:
        n_sampled = max(n_sampled, max(policy_w.t_stale + 1, args.warmup) + args.steps)
    t0 = time.time()
    if args.device_sampler:      # the mini-batches are sampled on the device below; the host samples only what the CPU oracle is timed on
        sampled = [] if args.no_cpu_baseline else sample_batches(w.name, 20, args.sample_workers)
    else:
        sampled = sample_batches(w.name, n_sampled, args.sample_workers)
    t_sample = time.time() - t0

    import numpy as np
    import torch
    from paper_2301_07482_amd.pipeline import DeviceBatch
    from paper_2301_07482_amd import pipeline as G

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    t0 = time.time()
    hot = buffer_bytes = None
    if args.feature_rows > 0:
        hot = wl.make_graph(w).hottest(args.feature_rows)
        row = w.feat_dim * (4 if w.feat_dtype == "f32" else 2)
        buffer_bytes = -(-(G.rings_bytes(w) + len(hot) * row) // 256) * 256
    hp, weights, feat = G.make_hotpath(w, use_cache=not args.no_cache, fused_input=not args.no_fuse, log_ring=total + extra + 32,
                                       hot_ids=hot, buffer_bytes=buffer_bytes, backward=args.backward, weight_grads=args.weight_grads, model=args.model,
                                       fetch_with_loader=not args.separate_fetch, admit_budget=admit_budget,
                                       overlap_update=not args.no_overlap_update, overlap_min_rows=65536,
                                       fuse_small_layers=not args.two_launch_seed_layer, copy_own_rows=args.copy_own_rows)
    ids_cols = not args.block_positions and not args.no_fuse
    make_batch = (lambda mb, gn, labels: DeviceBatch(mb, None, labels=labels, col_ids=ids_cols)) if args.backward else \
        (lambda mb, gn, labels: DeviceBatch(mb, gn, col_ids=ids_cols))
    if args.per_layer_update:
        hp.update_all = False
    if args.tune:
        from paper_2301_07482_amd import binding as B
        for kv in args.tune:
            key, value = kv.split("=")
            B.fg_set_tuning(key, int(value))
    sampler_report = {"where": "host", "workers": args.sample_workers, "seconds": t_sample, "minibatches": n_sampled,
                      "minibatches_per_s": n_sampled / t_sample if t_sample > 0 else None}
    if args.device_sampler:
        from fg_inputs import device as fdev, rng
        graph = wl.make_graph(w)
        t1 = time.time()
        indptr_t, indices_t = fdev.chunglu_csr(graph)
        t_csr = time.time() - t1
        ds = G.DeviceSampler(indptr_t, indices_t, w.num_nodes, w.fanouts, w.batch, transposes=args.backward)
        seeds = [torch.from_numpy(wl.seed_nodes(w, it).astype(np.int32)).cuda() for it in range(total + extra)]
        keys = [int(rng.make_key(w.seed, 0x5A3, it)) for it in range(total + extra)]
        ds.sample(seeds[0], keys[0])                      # first call: code objects, allocator
        outs = [ds.buffers() for _ in range(total + extra)]   # a consumer would recycle a few of these; here every mini-batch is kept
        torch.cuda.synchronize()
        for it in range(total + extra):                   # untimed pass: first use of the output memory
            ds.sample(seeds[it], keys[it], finish=False, out=outs[it])
        torch.cuda.synchronize()
        import gc
        gc.collect()
        gc.disable()      # keeping 100 mini-batch objects alive otherwise triggers a full collection inside the timed loop (30 ms)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t1 = time.time()
        e0.record()
        batches = [ds.sample(seeds[it], keys[it], finish=False, out=outs[it]) for it in range(total + extra)]   # no synchronisation per mini-batch
        e1.record()
        torch.cuda.synchronize()
        t_dev = time.time() - t1
        gc.enable()
        for b in batches:
            b.finish()
        sampler_report = {"where": "device", "minibatches": total + extra, "seconds": t_dev,
                          "ms_per_minibatch": 1e3 * t_dev / (total + extra), "minibatches_per_s": (total + extra) / t_dev,
                          "gpu_ms_per_minibatch": e0.elapsed_time(e1) / (total + extra), "csr_seconds": t_csr,
                          "csr_bytes": int(indptr_t.numel() * 8 + indices_t.numel() * 4),
                          "edges_per_minibatch": float(np.mean([sum(b.nnz) for b in batches]))}
        for it, b in enumerate(batches):                  # synthetic gradient norms by node id, as for host-sampled batches
            if args.backward:                             # ... or the seeds' classes, when the norms come from the backward pass
                b.labels = torch.from_numpy(wl.node_labels(w, wl.seed_nodes(w, it)).astype(np.int32)).cuda()
            else:
                b.gnorm = {l: torch.from_numpy(wl.grad_norms(w, it, l, b.ids[l][:b.n[l]].cpu().numpy())).cuda() for l in range(1, w.num_layers)}
        replay_batches = batches[total:]
        batches = batches[:total]
    else:
        batches = [make_batch(*s) for s in sampled[:total]]
    torch.cuda.synchronize()
    t_setup = time.time() - t0
    L = hp.L

    if args.calibration_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                     # reads 2**30 bytes, writes 2**30 bytes
        torch.cuda.synchronize()
        del a, b

    # untimed: prefill + warm-up. The last of these steps is given no look-ahead, so that the top-down pass of the first
    # timed mini-batch runs inside the timed region like that of every other timed step.
    for it in range(first_timed):
        hp.run(batches[it], it, next_bt=None if (args.no_lookahead or it + 1 == first_timed) else batches[it + 1])
    torch.cuda.synchronize()

    # timed region: exactly `steps` iterations. HIP events on the launch stream bracket only the two longest calls,
    # and only on every `--bracket-every`-th step, so that the region is not perturbed (an event record costs about
    # 3 us of stream time); the other calls are timed in a separate pass below.
    LOADER = "gather_features" if args.no_fuse else "gather_aggregate[1]"
    BRACKETED = (LOADER, "linear[1]")   # the two longest calls; whichever is longer is reported as `roofline`
    elapsed, timed_ms, timed_ovl_ms = timed_region(hp, batches, first_timed, args.steps, total, args.bracket_every,
                                                   not args.no_lookahead, BRACKETED)
    ms_per_step = 1e3 * elapsed / args.steps
    host_ms_per_step = 1e3 * timed_region.host_seconds / args.steps      # host time to queue a step's launches (below ms_per_step: the device is the bound)
    value = args.steps / elapsed

    # breakdown pass (not part of `value`): the iterations that follow the timed ones, on their own mini-batches, with
    # events around every call. It is a profile, not a result.
    ev2 = []
    replay_from_buffer = []
    replay = replay_batches if args.device_sampler else [make_batch(*sampled[total + k]) for k in range(extra)]
    overlapped = hp.overlap_update
    hp.overlap_update = False          # every call on the one stream here, so that each has a time of its own
    for k in range(extra):
        step_events = {}
        hp.run(replay[k], first_timed + args.steps + k, timer=timer_for(step_events))
        ev2.append(step_events)
        if hp.feature_side and args.no_fuse:   # the input list of this step, before the next one overwrites it
            ranks = torch.as_tensor(hp.feature_ranks(replay[k].ids[0], replay[k].n[0])[0], device="cuda")
            pos = hp.normal_pos[0][:int(hp.counts[0][2].item())].long()
            replay_from_buffer.append(float((ranks[pos] >= 0).sum().item()))
    torch.cuda.synchronize()
    hp.overlap_update = overlapped
    call_avg_ms = spans(ev2)

    counts_log = hp.counts_log.cpu().numpy()
    stats_log = hp.stats_log.cpu().numpy()
    steps_it = [first_timed + k for k in range(args.steps)]
    # the roofline figures price the launches that were bracketed: the same steps' counts
    roof_it = [first_timed + k for k in range(args.steps) if alone_step(k, args.steps, args.bracket_every)]
    counts = [counts_log[it % hp.ring] for it in roof_it]
    counts_all = [counts_log[it % hp.ring] for it in steps_it]
    esz = {"f32": 4, "f16": 2, "bf16": 2}
    # algorithmic bytes / flops per step, averaged over the timed steps
    feat_row = w.feat_dim * esz[w.feat_dtype]
    agg_row = w.feat_dim * (4 if w.compute_dtype == "f32" else 2)
    gather_bytes, n_input, dom_kernel = loader_bytes(hp, w, batches, roof_it, counts, not args.no_fuse, ids_cols, args.model)
    own_by_linear = hp.own_rows_from_table(batches[roof_it[0]])
    # rows the loader found on the feature side instead of reading them from the table (the placed rows lie beyond the
    # rings, so which nodes are there does not change during the run)
    from_buffer = 0.0
    if hp.feature_side:
        per_step = []
        for it in roof_it:
            bt = batches[it]
            ranks = torch.as_tensor(hp.feature_ranks(bt.ids[0], bt.n[0])[0], device="cuda")
            if args.no_fuse:       # counted on the steps of the breakdown pass
                per_step = replay_from_buffer
                break
            else:
                deg = (bt.end[1] - bt.start[1]).long()
                first = torch.repeat_interleave(bt.start[1].long(), deg)
                offs = torch.arange(int(deg.sum().item()), device="cuda") - torch.repeat_interleave(torch.cumsum(deg, 0) - deg, deg)
                src = bt.col[1].long()[first + offs]
                own = torch.nonzero(deg > 0).flatten()   # a lower bound of the normal rows (those left with neighbours)
                per_step.append(float((ranks[src] >= 0).sum().item() + (ranks[own] >= 0).sum().item()))
        from_buffer = float(np.mean(per_step))
    agg_bytes = {}
    lin_flops = {}
    lin_bytes = {}
    for l in range(1, L + 1):
        d_in, d_out = hp.dims[l - 1], hp.dims[l]
        e_in = 4 if (l == 1 and w.feat_dtype == "f32") or w.compute_dtype == "f32" else 2
        nn = float(np.mean([c[l][2] for c in counts]))
        k_l = d_in if args.model == "gcn" else 2 * d_in       # contraction length of the dense update
        lin_flops[l] = 2.0 * nn * k_l * d_out
        lin_bytes[l] = nn * (k_l * e_in + d_out * 4) + k_l * d_out * 4
    dom = max(call_avg_ms, key=call_avg_ms.get)
    gather_ms = timed_ms[LOADER]
    if w.feat_location == "host":
        # host-resident table: the loader is bound by the host link, priced on the table bytes that cross it
        link_bytes = (n_input - from_buffer) * feat_row
        loader_roof = dict(bound="host_link", kernel=dom_kernel, achieved=link_bytes / (gather_ms * 1e-3) / 1e9,
                           peak=PCIE5_X16_GBS, unit="GB/s", frac=link_bytes / (gather_ms * 1e-3) / 1e9 / PCIE5_X16_GBS,
                           traffic=None, bytes_per_launch=link_bytes, ms_per_launch=gather_ms)
    else:
        loader_roof = dict(bound="hbm", kernel=dom_kernel,
                           achieved=gather_bytes / (gather_ms * 1e-3) / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
                           frac=gather_bytes / (gather_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, traffic=None,
                           bytes_per_launch=gather_bytes, ms_per_launch=gather_ms)
    lin1_ms = timed_ms["linear[1]"]
    # The layer-1 dense update is an fp32 contraction (fp32 operands and result, fp32/fp64 accumulation) priced against
    # the fp32 matrix peak on its algorithmic flops 2*M*K*N. Its default kernel forms every fp32 product exactly from
    # three bf16 pieces per operand (6 partial products on v_mfma_f32_32x32x16_bf16), so the matrix cores execute 6x
    # the algorithmic flops at the bf16 rate: that figure is given as well.
    lin_tf = lin_flops[1] / (lin1_ms * 1e-3) / 1e12
    if w.compute_dtype == "bf16":
        linear_roof = dict(bound="mfma", kernel="linear_bf16_kernel (fg_linear, layer 1, bf16 MFMA, fp32 accumulation)",
                           achieved=lin_tf, peak=BF16_MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=lin_tf / BF16_MFMA_PEAK_TFLOPS,
                           traffic=None, flops_per_launch=lin_flops[1], ms_per_launch=lin1_ms)
    elif (hp.dims[0] // 2 if args.model == "gcn" else hp.dims[0]) % 32 == 0:
        linear_roof = dict(bound="mfma", kernel="linear_f32x3_panel_kernel<2> (fg_linear, layer 1: fp32 products from 3-way bf16 "
                                                "splits on the bf16 matrix cores)",
                           achieved=lin_tf, peak=FP32_MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=lin_tf / FP32_MFMA_PEAK_TFLOPS,
                           traffic=None, flops_per_launch=lin_flops[1], ms_per_launch=lin1_ms,
                           executed=dict(tflops=6 * lin_tf, peak=BF16_MFMA_PEAK_TFLOPS, frac=6 * lin_tf / BF16_MFMA_PEAK_TFLOPS,
                                         note="bf16 MFMA flops issued (6 partial products per fp32 product)"))
    else:  # input width not a multiple of 32: the LDS-tiled fp32-MFMA kernel
        linear_roof = dict(bound="mfma", kernel="linear_f32_kernel (fg_linear, layer 1, fp32 MFMA)",
                           achieved=lin_tf, peak=FP32_MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=lin_tf / FP32_MFMA_PEAK_TFLOPS,
                           traffic=None, flops_per_launch=lin_flops[1], ms_per_launch=lin1_ms)
    if w.name == "large_hbm" and not (args.no_cache or args.no_fuse or args.model != "sage" or args.feature_rows):   # the configuration the counter runs were made on
        loader_roof["traffic"] = profiled_traffic("loader_fetch_kernel<0, 0>" if dom_kernel.startswith("loader_fetch") else "aggregate_mean_kernel<0, 0, true, false")
        linear_roof["traffic"] = profiled_traffic("linear_f32x3_panel_kernel<2>")
        for r in (loader_roof, linear_roof):      # not measured in this run: counters need the profiler around the process
            r["traffic_source"] = ("profiles/bench_large_hbm_hbm_traffic.md: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                   "command, committed with the code") if r["traffic"] is not None else None
    # `roofline` is the kernel with the longest launches in the timed region; the other one follows as `roofline_2`
    if LOADER in timed_ovl_ms:       # the same launches as they run in most steps, beside the second stream's bookkeeping
        loader_roof["ms_per_launch_overlapped"] = timed_ovl_ms[LOADER]
        linear_roof["ms_per_launch_overlapped"] = timed_ovl_ms.get("linear[1]")
    roofline, roofline_2 = (loader_roof, linear_roof) if gather_ms >= lin1_ms else (linear_roof, loader_roof)

    hits = {l: float(np.mean([c[l][1] for c in counts_all])) for l in range(1, L)}
    n0_all = float(np.mean([batches[it].n[0] for it in steps_it]))

    # Everything but the dense updates (lookup, prune, compaction, fetch, loader, aggregation, update) as one
    # bandwidth figure: algorithmic bytes of those steps over the time of their calls in the breakdown pass.
    stats = [stats_log[it % hp.ring] for it in roof_it]
    e_comp = 4 if w.compute_dtype == "f32" else 2
    def call_bytes(it, c, st):
        """Algorithmic bytes of every call of one step except the loader and the dense updates, keyed like per_call_ms."""
        out = {}
        add = lambda k, v: out.__setitem__(k, out.get(k, 0.0) + v)
        for l in range(1, L + 1):
            n_l, n_hit, n_norm = batches[it].n[l], float(c[l][1]), float(c[l][2])
            edges_l = float((batches[it].end[l] - batches[it].start[l]).sum().item())      # left under normal rows
            add("top_down", n_l * (4 + 1 + 4 + 8) + edges_l * (4 + 1) + 4 * (2 * n_hit + n_norm))   # lookup, prune, lists
            if l >= 2 or args.no_fuse:
                d_prev = hp.dims[l - 1] * (esz[w.feat_dtype] if l == 1 else e_comp)
                add(f"aggregate[{l}]", edges_l * (4 + d_prev) + n_norm * hp.dims[l - 1] * e_comp)
            if l < L:
                row = hp.dims[l] * e_comp
                if "cache_fetch_all" in call_avg_ms:      # otherwise counted with the loader, whose launch does it
                    add("cache_fetch_all", n_hit * (8 + 2 * row))
                add("cache_update_all", 2 * n_l * 6 + float(st[l][0]) * (2 * row + 12) + float(st[l][1]) * 4)
        return out
    per_step_bytes = [call_bytes(it, c, st) for it, c, st in zip(roof_it, counts, stats)]
    call_avg_bytes = {k: float(np.mean([d.get(k, 0.0) for d in per_step_bytes])) for k in per_step_bytes[0]} if per_step_bytes else {}
    # a small layer that runs aggregation and dense update as one launch counts as a dense call (its means never reach memory)
    one_launch = [int(k[len("aggregate_linear["):-1]) for k in call_avg_ms if k.startswith("aggregate_linear[")]
    for l in one_launch:
        call_avg_bytes.pop(f"aggregate[{l}]", None)
    path_bytes = gather_bytes + sum(call_avg_bytes.values())
    call_avg_bytes[LOADER] = gather_bytes
    # every call: time in the breakdown pass, algorithmic bytes (or flops) and the rate they give
    per_call = {}
    for k, ms in sorted(call_avg_ms.items()):
        e = {"ms": round(ms, 5)}
        if k in call_avg_bytes and ms > 0:
            e.update(bytes=call_avg_bytes[k], GBps=round(call_avg_bytes[k] / (ms * 1e-3) / 1e9, 1))
        elif k.startswith(("linear[", "aggregate_linear[")) and ms > 0:
            f = lin_flops[int(k[k.index("[") + 1:-1])]
            e.update(flops=f, TFLOPs=round(f / (ms * 1e-3) / 1e12, 1))
        per_call[k] = e
    path_ms = sum(v for k, v in call_avg_ms.items() if not k.startswith(("linear", "aggregate_linear", "loss_grad", "layer_backward", "row_norms", "weight_grads")))
    hbm_path = dict(bytes_per_step=path_bytes, ms_per_step=path_ms, achieved=path_bytes / (path_ms * 1e-3) / 1e9, peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=path_bytes / (path_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    note="all calls except the dense updates (fg_linear, fg_aggregate_linear); times from the breakdown pass (every call bracketed)")
    # The benchmark spec's figure: lookup + prune + compaction + cache fetch + feature gather + aggregation (steps a1-a6 of the
    # path: everything up to the dense updates, without the cache update), algorithmic bytes over the time of those calls
    # in the breakdown pass, where every call runs on the one stream and has a time of its own.
    a1_a6 = [k for k in call_avg_ms if k.startswith(("top_down", "lookup_prune", "gather_features", "gather_aggregate", "cache_fetch", "aggregate["))]
    a1_a6_bytes = sum(call_avg_bytes.get(k, 0.0) for k in a1_a6)
    a1_a6_ms = sum(call_avg_ms[k] for k in a1_a6)
    path_a1_a6 = dict(bound="hbm", bytes=a1_a6_bytes, ms=a1_a6_ms, achieved=a1_a6_bytes / (a1_a6_ms * 1e-3) / 1e9 if a1_a6_ms else None,
                      peak=HBM_PEAK_GBS, unit="GB/s", frac=a1_a6_bytes / (a1_a6_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if a1_a6_ms else None,
                      calls=sorted(a1_a6), target_frac=0.60,
                      note="lookup+gather+aggregate path (top-down pass, loader with the cache fetch, aggregations of the upper "
                           "layers; aggregations that run inside a dense update's launch are counted with that update), one stream, every call bracketed")
    # table rows the loader would read with the caches empty: every edge of block 1 plus every layer-1 node's own row
    if args.no_fuse:
        rows_no_cache = n0_all
    else:
        rows_no_cache = float(np.mean([batches[it].nnz[1] + batches[it].n[1] for it in steps_it]))

    if args.device_sampler:      # the loop with nothing resident beforehand but the graph, the table and the seeds
        sampler_report["in_loop"] = sampled_loop(w, hp, ds, first_it=total + extra, steps=args.steps, warmup=10, backward=args.backward,
                                                 lookahead=not args.no_lookahead)
        sampler_report["in_loop_host_sizes"] = sampled_loop(w, hp, ds, first_it=total + extra + args.steps + 10, steps=args.steps, warmup=10,
                                                            backward=args.backward, lookahead=not args.no_lookahead, host_sizes=True)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = time_oracle(w, sampled, weights)

    hp.close()
    policy_paper = None
    if policy_w is not None:
        del batches, replay
        torch.cuda.empty_cache()
        policy_paper = policy_paper_run(policy_w, feat, sampled, args, ids_cols)
    out = {
        "metric": "sampled mini-batches/sec (lookup+gather+aggregate+update); achieved GB/s vs roofline",
        "value": value, "unit": "mini-batches/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.compute_dtype == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": w.name, "num_nodes": w.num_nodes, "num_edges": w.num_edges, "feat_dim": w.feat_dim,
                   "feat_dtype": w.feat_dtype, "features": w.feat_location, "layers": L, "hidden": w.hidden,
                   "fanouts": list(w.fanouts), "batch": w.batch, "cache_slots_per_layer": w.cache_capacity,
                   "t_stale": w.t_stale, "p_grad": w.p_grad, "cache": not args.no_cache,
                   "fused_loader": not args.no_fuse, "feature_rows": int(args.feature_rows),
                   "gradient_norms": "backward pass" if args.backward else "synthetic input",
                   "weight_gradients": bool(args.weight_grads and args.backward), "layer_type": args.model,
                   "top_down": "of the next mini-batch on the second stream, beside this step's layers" if (
                       not args.no_lookahead and hp.overlap_update and not args.backward and not args.no_cache and not args.per_layer_update
                       and not hp.feature_side and hp.one_launch_top_down) else "at the start of the step",
                   "update_selection": "second stream, beside the layers" if (hp.overlap_update and not args.backward and not args.no_cache
                                                                              and not args.per_layer_update and not hp.feature_side) else "after the layers",
                   "block1_columns": "node ids" if ids_cols else "positions",
                   "own_rows_layer1": "read from the table by the dense update (fg_linear_ids)" if own_by_linear
                   else "copied out by the loader", "seed": w.seed},
        "prefill_steps": prefill,
        "roofline": roofline,
        "roofline_2": roofline_2,
        "path_a1_a6": path_a1_a6,
        "policy_paper": policy_paper,
        "cpu_baseline": cpu_baseline,
        "per_call_ms": {k: round(v, 5) for k, v in sorted(call_avg_ms.items())},
        "per_call": per_call,
        "dominant_call": dom,
        "hbm_path": hbm_path,
        "per_step": {"table_rows_read": n_input - from_buffer, "rows_from_feature_side": from_buffer,
                     "table_rows_without_cache": rows_no_cache,
                     "io_saving": 1.0 - (n_input - from_buffer) / rows_no_cache if rows_no_cache else 0.0,
                     "io_saving_embeddings_only": 1.0 - n_input / rows_no_cache if rows_no_cache else 0.0,
                     "input_rows_sampled": n0_all,
                     "hits": hits, "gather_bytes": gather_bytes, "linear_flops": lin_flops},
        "admit_budget": admit_budget,
        "sampler": sampler_report,
        "host": {"sampling_s": t_sample, "setup_s": t_setup, "queueing_ms_per_step": host_ms_per_step},
    }
    print(json.dumps(out))


def timer_for(step_events, only=None):
    """A `timer` for HotPath.run that records a HIP event (on the stream the call is launched on) before each call named
    in `only` (every call if None) and after it."""
    import torch
    is_open = {}

    def tick(name, stream=None):
        key = id(stream) if stream is not None else 0
        if only is not None:
            if not (name in only or is_open.get(key, False)):
                return
            is_open[key] = name in only
        e = torch.cuda.Event(enable_timing=True)
        e.record(stream) if stream is not None else e.record()
        step_events.setdefault(key, []).append((name, e))
    return tick


def spans(event_log):
    """Mean time of every bracketed call over the steps of an event log, ms."""
    import numpy as np
    out = {}
    for step_events in event_log:
        for per_stream in step_events.values():
            for (name, e0), (_, e1) in zip(per_stream[:-1], per_stream[1:]):
                if name is not None:
                    out.setdefault(name, []).append(e0.elapsed_time(e1))
    return {k: float(np.mean(v)) for k, v in out.items()}


def alone_step(k, steps, bracket_every):
    """Whether timed step k is one whose bracketed launches have the chip to themselves: every `bracket_every`-th step,
    starting half a period in (the first step after the opening synchronisation finds an idle device and is no sample
    of the steady state); step 0 where the region is shorter than that."""
    first = bracket_every // 2 if steps > bracket_every // 2 else 0
    return k >= first and (k - first) % bracket_every == 0


def timed_region(hp, batches, first_timed, steps, total, bracket_every, lookahead, bracketed):
    """Exactly `steps` iterations (mini-batches first_timed ..) between two device synchronisations. HIP events on the
    launch stream bracket only the calls named in `bracketed`, and only on every `bracket_every`-th step, so that the
    region is not perturbed (an event record costs about 3 us of stream time). Two kinds of bracketed steps: in every
    `bracket_every`-th step the bracketed launches have the chip to themselves (the durations `roofline` is priced on,
    comparable with a kernel trace; the first of these steps comes half a period into the region, see alone_step): the
    second stream's bookkeeping of that step is held back until layer 1 is done, or, where the pipeline has nothing to
    hold (backward pass, feature side), every call of the step runs on the one stream; half way between them a step is
    bracketed as it normally runs, with the bookkeeping launches of the second stream beside it.
    Returns (seconds, {call: ms} of the one-stream steps, {call: ms} of the overlapped steps)."""
    import torch
    ev, ev_ovl = [], []
    overlapped = hp.overlap_update
    can_hold = hp.holds_second_stream()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(steps):
        it = first_timed + k
        step_events = {}
        alone = alone_step(k, steps, bracket_every)
        beside = overlapped and k > 0 and k % bracket_every == 0
        ahead = batches[it + 1] if (it + 1 < total and lookahead and (can_hold or not alone)) else None   # its top-down pass runs beside this step's layers
        if not can_hold:
            hp.overlap_update = overlapped and not alone
        hp.run(batches[it], it, timer=timer_for(step_events, only=bracketed) if (alone or beside) else None, next_bt=ahead,
               hold_second_stream=alone and can_hold)
        (ev if alone else ev_ovl).append(step_events)
    hp.flush()      # the last step's row copy (left to the next call when that call's top-down pass is already queued) belongs to it
    t_queued = time.perf_counter()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    hp.overlap_update = overlapped
    timed_region.host_seconds = t_queued - t_start      # the host's own share: every launch of the region is queued by then
    return elapsed, spans(ev), spans(ev_ovl)


def loader_bytes(hp, w, batches, its, counts, fused, ids_cols, model):
    """Algorithmic bytes per launch of the loader, averaged over the iterations `its` (their device-side counts in
    `counts`), the table rows it reads, and the kernel's name."""
    import numpy as np
    esz = {"f32": 4, "f16": 2, "bf16": 2}
    L = hp.L
    feat_row = w.feat_dim * esz[w.feat_dtype]
    agg_row = w.feat_dim * (4 if w.compute_dtype == "f32" else 2)
    if not fused:
        # feature gather: per gathered row 4 (id) + row read + row written
        gather_bytes = float(np.mean([c[0][2] * (4 + 2 * feat_row) for c in counts]))
        n_input = float(np.mean([c[0][2] for c in counts]))
        return gather_bytes, n_input, "gather_rows_kernel<.., true> (fg_gather of the raw features)"
    # fused loader + layer-1 mean: per edge of a normal row 4 (col) [+ 4 (id) when the block's columns are positions] + one
    # table row read; per normal row 4 (position) + 8 (start, end) + one mean row written + its own row: 4 (id) + one
    # table row read + one row written. The edges under normal rows are what is left in the pruned blocks (rows that are
    # not normal have end = start).
    edges = [float((batches[it].end[1] - batches[it].start[1]).sum().item()) for it in its]
    own_row = (4 + feat_row) if model == "gcn" else (4 + 2 * feat_row)   # GCN: the own row enters the mean, no copy
    own_by_linear = hp.own_rows_from_table(batches[its[0]])               # the dense update reads the own rows itself
    if own_by_linear:
        own_row = 0
    per_edge = (4 if ids_cols and not hp.feature_side and model == "sage" else 8) + feat_row   # column (+ position -> id) + row
    gather_bytes = float(np.mean([e * per_edge + c[1][2] * (12 + agg_row + own_row) for e, c in zip(edges, counts)]))
    # table rows read (edges + own rows: the latter by the loader, or by the dense update of layer 1)
    n_input = float(np.mean(edges)) + float(np.mean([c[1][2] for c in counts]))
    kernel = "aggregate_mean_kernel<.., true> (fg_gather_aggregate: loader fused with the layer-1 mean)"
    fetch_rides = (ids_cols and hp.fetch_with_loader and hp.fetch_all and hp.cache is not None and hp.use_cache
                   and model == "sage" and not hp.feature_side and not hp.one_launch(1, batches[its[0]].n[1]))
    if fetch_rides:   # the launch also fetches the cached embeddings: per hit 8 (slot, position) + a row read + a row written
        e_c = 4 if w.compute_dtype == "f32" else 2
        gather_bytes += float(np.mean([sum(c[l][1] * (8 + 2 * hp.dims[l] * e_c) for l in range(1, L)) for c in counts]))
        kernel = "loader_fetch_kernel (fg_gather_aggregate_ids: loader fused with the layer-1 mean, cache fetch in the same launch)"
    return gather_bytes, n_input, kernel


def policy_paper_run(w, feat, sampled, args, ids_cols):
    """The same path with the paper's default thresholds (Section 7.1: t_stale 200, p_grad 0.9) instead of the workload's,
    on a cache of its own that is first brought to its steady state (t_stale + 1 untimed iterations): throughput, what
    the pruning saves, and the loader's roofline figures, measured like the headline's."""
    import numpy as np
    import torch
    from paper_2301_07482_amd import pipeline as G
    from paper_2301_07482_amd.pipeline import DeviceBatch
    first_timed = max(w.t_stale + 1, args.warmup)
    total = first_timed + args.steps
    fused = not args.no_fuse
    hp, _, _ = G.make_hotpath(w, feat_table=feat, fused_input=fused, log_ring=total + 32, model=args.model,
                              fetch_with_loader=not args.separate_fetch, overlap_update=not args.no_overlap_update,
                              overlap_min_rows=65536, fuse_small_layers=not args.two_launch_seed_layer, copy_own_rows=args.copy_own_rows)
    try:
        batches = [DeviceBatch(mb, gn, col_ids=ids_cols) for mb, gn, _ in sampled[:total]]
        for it in range(first_timed):
            hp.run(batches[it], it, next_bt=None if (args.no_lookahead or it + 1 == first_timed) else batches[it + 1])
        loader = "gather_aggregate[1]" if fused else "gather_features"
        elapsed, timed_ms, _ = timed_region(hp, batches, first_timed, args.steps, total, args.bracket_every, not args.no_lookahead,
                                            (loader, "linear[1]"))
        counts_log = hp.counts_log.cpu().numpy()
        roof_it = [first_timed + k for k in range(args.steps) if alone_step(k, args.steps, args.bracket_every)]
        steps_it = [first_timed + k for k in range(args.steps)]
        counts = [counts_log[it % hp.ring] for it in roof_it]
        counts_all = [counts_log[it % hp.ring] for it in steps_it]
        nbytes, _, kernel = loader_bytes(hp, w, batches, roof_it, counts, fused, ids_cols, args.model)
        _, rows_read, _ = loader_bytes(hp, w, batches, steps_it, counts_all, fused, ids_cols, args.model)
        if fused:
            rows_no_cache = float(np.mean([batches[it].nnz[1] + batches[it].n[1] for it in steps_it]))
        else:
            rows_no_cache = float(np.mean([batches[it].n[0] for it in steps_it]))
        ms = timed_ms[loader]
        on_host = w.feat_location == "host"
        esz = {"f32": 4, "f16": 2, "bf16": 2}
        moved = rows_read * w.feat_dim * esz[w.feat_dtype] if on_host else nbytes
        peak = PCIE5_X16_GBS if on_host else HBM_PEAK_GBS
        return {"t_stale": w.t_stale, "p_grad": w.p_grad, "prefill_steps": first_timed - args.warmup, "warmup": args.warmup,
                "steps": args.steps, "value": args.steps / elapsed, "unit": "mini-batches/s", "ms_per_step": 1e3 * elapsed / args.steps,
                "io_saving": 1.0 - rows_read / rows_no_cache if rows_no_cache else 0.0,
                "table_rows_read": rows_read, "table_rows_without_cache": rows_no_cache,
                "hits": {l: float(np.mean([c[l][1] for c in counts_all])) for l in range(1, hp.L)},
                "roofline": {"bound": "host_link" if on_host else "hbm", "kernel": kernel, "achieved": moved / (ms * 1e-3) / 1e9,
                             "peak": peak, "unit": "GB/s", "frac": moved / (ms * 1e-3) / 1e9 / peak, "traffic": None,
                             "bytes_per_launch": moved, "ms_per_launch": ms},
                "note": "the paper's default thresholds on the same workload, same kernels and launch configuration"}
    finally:
        hp.close()
        del hp
        torch.cuda.empty_cache()


def sampled_loop(w, hp, ds, first_it, steps, warmup, backward=False, lookahead=True, host_sizes=False):
    """Iterations whose mini-batches are sampled on the device while the loop runs: the sampler works two mini-batches ahead
    on a second stream, gradient norms are made on the device from the sampled node ids, and the path's stream waits for
    the sampler's event. The layer sizes stay in device memory (the calls get the sampler's bounds and the addresses of the
    counts), so the host never waits for the device inside the loop; host_sizes=True is the variant in which the sizes
    reach the host through a pinned copy and the host waits for each mini-batch's event. Four sets of buffers rotate."""
    import torch
    from fg_inputs import device as fdev, rng, workload as wl
    L, K = w.num_layers, 4
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    outs = [ds.buffers() for _ in range(K)]
    gn = [{l: torch.empty(ds.bound[l], dtype=torch.float32, device="cuda") for l in range(1, L)} for _ in range(K)]
    host_counts = [torch.zeros((L + 1, 2), dtype=torch.int64, pin_memory=True) for _ in range(K)]
    sampled_ev = [torch.cuda.Event() for _ in range(K)]
    consumed_ev = [torch.cuda.Event() for _ in range(K)]
    n_it = warmup + steps
    seeds = [torch.from_numpy(wl.seed_nodes(w, first_it + t).astype("int32")).cuda() for t in range(n_it)]
    keys = [int(rng.make_key(w.seed, 0x5A3, first_it + t)) for t in range(n_it)]
    gkeys = [{l: int(rng.make_key(w.seed, 0x6AD, first_it + t, l)) for l in range(1, L)} for t in range(n_it)]
    labels = [torch.from_numpy(wl.node_labels(w, wl.seed_nodes(w, first_it + t)).astype("int32")).cuda() for t in range(n_it)] if backward else None
    torch.cuda.synchronize()

    def launch(t):
        k = t % K
        with torch.cuda.stream(side):
            if t >= K:
                side.wait_event(consumed_ev[k])        # the path is done with this set of buffers
            bt = ds.sample(seeds[t], keys[t], finish=False, out=outs[k], ready=False)
            if backward:          # the norms come from the backward pass; it needs the seeds' classes
                bt.labels = labels[t]
            else:
                for l in range(1, L):
                    fdev.grad_norms(bt.ids[l], bt._counts.data_ptr() + 16 * l, ds.bound[l], gkeys[t][l], gn[k][l], side.cuda_stream)
                bt.gnorm = gn[k]
            if host_sizes:
                host_counts[k].copy_(bt._counts, non_blocking=True)
            sampled_ev[k].record(side)
            bt.ready = sampled_ev[k]       # behind the norms as well: what the path's second stream waits for
        return bt

    def ready(t, bt):
        """Mini-batch t as the path takes it (host_sizes: with its layer sizes on the host)."""
        k = t % K
        if host_sizes:
            sampled_ev[k].synchronize()
            bt.finish(host_counts[k])
        return bt      # (its `ready` event orders the path's streams behind the sampling: HotPath.run)

    # the sampler works two mini-batches ahead, so that the next one is complete (sizes known) when this one is run and
    # its top-down pass can go to the second stream beside this one's layers
    queue = {0: launch(0)}
    if n_it > 1:
        queue[1] = launch(1)
    cur = ready(0, queue.pop(0))
    t_start = None
    for t in range(n_it):
        if t == warmup:
            torch.cuda.synchronize()
            t_start = time.time()
        if t + 2 < n_it:
            queue[t + 2] = launch(t + 2)
        nxt = ready(t + 1, queue.pop(t + 1)) if t + 1 < n_it else None
        hp.run(cur, first_it + t, next_bt=nxt if lookahead else None)
        # the buffers of mini-batch t - 1 are free once this call's launches are through: the call started behind the second
        # stream's last reads of that mini-batch (its update's selection), and its own launches follow the row copy
        if t >= 1:
            consumed_ev[(t - 1) % K].record(main)
        cur = nxt
    t_queued = time.time()      # everything is queued: the host's own share of the loop
    torch.cuda.synchronize()
    dt = time.time() - t_start
    return {"steps": steps, "warmup": warmup, "ms_per_step": 1e3 * dt / steps, "minibatches_per_s": steps / dt,
            "host_ms_per_step": 1e3 * (t_queued - t_start) / steps,
            "host_synchronisations_per_minibatch": 1 if host_sizes else 0,
            "note": "sampling (a stream of its own, two mini-batches ahead), gradient norms and the whole path inside the timed loop; "
                    + ("layer sizes read back through a pinned copy" if host_sizes else "layer sizes never leave the device")}


def profiled_traffic(kernel_prefix):
    """HBM bytes per launch of a kernel from the committed rocprofv3 counter summary (FETCH_SIZE and WRITE_SIZE runs of
    this same command, scaled by the plain-copy calibration stated there); None if the summary has no such row."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "bench_large_hbm_hbm_traffic.md")
    try:
        for line in open(path):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 5 and cells[0].startswith(kernel_prefix):
                return (float(cells[3]) + float(cells[4])) * 1e6
    except (OSError, ValueError):
        pass
    return None


def cpu_model():
    """Model name of the host's processor as /proc/cpuinfo gives it."""
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return None


def time_oracle(w, sampled, weights, iterations=20):
    """The CPU oracle timed on the first `iterations` mini-batches of the same workload (from an empty cache),
    single-threaded; feature rows are regenerated beforehand and not timed."""
    import numpy as np
    from fg_inputs import features, workload as wl
    from oracle import freshgnn_oracle as O
    from tests import gpu_common as G      # builds the oracle's caches: used by this leg only
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:  # pragma: no cover
        limiter = None
    caches = G.make_oracle_caches(w)
    dims = wl.layer_dims(w)
    dt = np.float32 if w.feat_dtype == "f32" else np.float16
    secs = 0.0
    done = 0
    for it in range(min(iterations, len(sampled))):
        mb, gn = sampled[it][:2]
        mb = mb.copy()
        rows = features.feature_rows(w.seed, mb.ids[0], w.feat_dim, dt)      # not timed: input generation
        order = np.argsort(mb.ids[0], kind="stable")
        sorted_ids = mb.ids[0][order]

        def frows(ids, rows=rows, order=order, sorted_ids=sorted_ids):
            return rows[order[np.searchsorted(sorted_ids, ids)]]

        t0 = time.perf_counter()
        O.iteration(mb, it, caches, frows, weights, gn, w.p_grad, dims, w.feat_dtype, w.compute_dtype)
        secs += time.perf_counter() - t0
        done += 1
        if secs > 20.0:
            break
    if limiter is not None:
        limiter.restore_original_limits()
    return {"value": done / secs, "unit": "mini-batches/s", "cores": 1, "cpu_model": cpu_model(), "host_cores": os.cpu_count(),
            "kind": "oracle",
            "sample": f"iterations 0..{done - 1} of the same workload from an empty cache, {secs:.1f} s of CPU time, "
                      "feature-row generation excluded"}


if __name__ == "__main__":
    main()
