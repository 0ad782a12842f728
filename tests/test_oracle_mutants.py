"""Do the pins of the oracle bite? Each case plants one plausible mistake in the oracle (a dropped term, a wrong
sign or bound, swapped operands), on the CPU, and requires that at least one pin of test_oracle_pins.py then fails.
The mistakes are made by editing the source text of one oracle function and re-executing it in the oracle module."""
import inspect
import textwrap

import pytest

from oracle import freshgnn_oracle as O
from tests import test_oracle_access_policy as AP
from tests import test_oracle_backward as BW
from tests import test_oracle_feature_side as F
from tests import test_oracle_mixed_precision as MP
from tests import test_oracle_pins as P

PINS = [
    (P.test_full_neighbourhood_equals_dense_recursion, [(1, 0), (2, 1), (3, 2)]),
    (P.test_intermediate_layers_equal_dense_recursion, [()]),
    (P.test_mean_closed_forms, [()]),
    (P.test_linear_panels_and_activation, [()]),
    (P.test_bf16_rounding_points, [()]),
    (P.test_prune_matches_depth_first_needed_set, [(s,) for s in range(4)]),
    (P.test_exact_history_invariant, [()]),
    (P.test_degenerate_settings_reduce_to_neighbour_sampling, [(0.0, 5), (0.7, 0)]),
    (P.test_admit_everything_keeps_everything_computed, [()]),
    (P.test_threshold_is_rank_statistic_and_order_free, [()]),
    (P.test_trace_gradient_and_staleness, [()]),
    (P.test_trace_ring, [()]),
    (P.test_staleness_boundary, [()]),
    (P.test_cache_matches_dictionary_model, [(5, 2, 0.5), (16, 4, 0.9), (3, 1, 1.0), (40, 50, 0.3)]),
    (P.test_stabilization_period_is_plain_sampling_then_a_cache_that_starts_empty, [()]),
    (P.test_gcn_full_neighbourhood_equals_dense_recursion_and_closed_forms, [()]),
    (F.test_trace_junction, [()]),
    (F.test_validity_equals_untouched_bytes_and_rows_stay_bit_identical,
     [(0, "f32", "f32", 4096, [5, 3], [12, 20], 8, 128), (1, "f32", "f32", 8192, [7, 4], [36, 8], 12, 170),
      (2, "bf16", "f16", 4096, [9, 6], [24, 40], 24, 85), (4, "f32", "f32", 2048, [3, 2, 2], [8, 8, 8], 8, 10)]),
    (F.test_ring_rows_are_laid_down_in_the_shared_buffer, [()]),
    (F.test_one_ring_keeps_a_prefix_of_the_hot_list, [()]),
    (F.test_hot_order_properties, [()]),
    (F.test_feature_side_changes_where_rows_come_from_and_nothing_else, [()]),
    (BW.test_loss_gradient_against_finite_differences_and_row_sums, [()]),
    (BW.test_row_norms, [()]),
    (BW.test_embedding_gradients_against_finite_differences, [(2, 0), (3, 1), (3, 2)]),
    (BW.test_weight_gradients_against_finite_differences, [()]),
    (BW.test_gradient_norms_from_the_backward_pass_drive_the_update, [()]),
    (AP.test_estimate_counts_the_rows_an_unshared_evaluation_reads, [(0,), (1,), (2,)]),
    (AP.test_estimate_on_full_trees_is_a_product_and_saturates, [()]),
    (AP.test_estimate_hand_example, [()]),
    (AP.test_admission_hand_example, [()]),
    (AP.test_admission_is_the_rank_definition, [(0,), (1,), (2,)]),
    (AP.test_without_estimates_and_budget_nothing_changes, [(5, 2, 0.5), (16, 4, 0.9)]),
    (AP.test_iteration_with_budget_admits_the_costliest_rows, [()]),
    (MP.test_worked_example_of_the_rounding_points, [()]),
    (MP.test_identity_panels_show_each_rounded_operand_bit_for_bit, [(0,), (1,)]),
    (MP.test_products_take_bf16_operands_and_the_last_layer_keeps_fp32, [()]),
    (MP.test_cached_rows_are_bf16_and_fetched_bit_for_bit, [()]),
    (MP.test_backward_rounds_the_output_gradient_before_both_products, [()]),
    (MP.test_backward_of_a_lower_layer_masks_then_rounds_and_uses_rounded_weights, [()]),
    (MP.test_gcn_gradients_against_finite_differences, [(0,), (1,)]),
]

# (owner, function, text in its source, replacement)
MUTANTS = [
    ("aggregate sums instead of averaging", None, "aggregate", "/ float(len(nb))", "/ 1.0"),
    ("aggregate divides by degree + 1", None, "aggregate", "/ float(len(nb))", "/ float(len(nb) + 1)"),
    ("aggregate reads rows instead of neighbours", None, "aggregate", "h[nb]", "h[[r] * len(nb)]"),
    ("linear swaps the self and neighbour panels", None, "linear", "@ W[:d_in] + np.asarray(agg, dtype=np.float64) @ W[d_in:]",
     "@ W[d_in:] + np.asarray(agg, dtype=np.float64) @ W[:d_in]"),
    ("linear drops the bias", None, "linear", "+ np.asarray(b, dtype=np.float64))", "+ 0.0 * np.asarray(b, dtype=np.float64))"),
    ("linear applies ReLU after the last layer too", None, "linear", "if relu else z", "if True else z"),
    ("linear never applies ReLU", None, "linear", "if relu else z", "if False else z"),
    ("an entry is usable in the iteration that admitted it", "HistoricalCache", "slot_of", "age < 1", "age < 0"),
    ("staleness bound one too short", "HistoricalCache", "slot_of", "age > self.t_stale", "age >= self.t_stale"),
    ("staleness bound one too long", "HistoricalCache", "slot_of", "age > self.t_stale", "age > self.t_stale + 1"),
    ("recycled slots still hit for their old owner", "HistoricalCache", "slot_of", "int(self.slot_node[s]) != int(v)", "False"),
    ("threshold rank one too low", None, "admission_threshold", "[k]), k", "[k - 1]), k"),
    ("threshold count rounds up", None, "admission_threshold", "np.floor(", "np.ceil("),
    ("ties at the threshold are admitted", None, "cache_update", "not hit[j] and g[j] < tau", "not hit[j] and g[j] <= tau"),
    ("hits with large norms are kept", None, "cache_update", "cache.map[ids[j]] = -1", "pass"),
    ("hits at the threshold are kept", None, "cache_update", "hit[j] and not (g[j] < tau)", "hit[j] and not (g[j] <= tau)"),
    ("population of the percentile is the computed nodes only", None, "cache_update", "admission_threshold(g[live], p_grad)",
     "admission_threshold(g[live & ~hit], p_grad)"),
    ("admitted rows are stamped with the next iteration", None, "cache_update", "cache.slot_stamp[s] = i", "cache.slot_stamp[s] = i + 1"),
    ("the ring header does not advance", None, "cache_update", "cache.head = (head + admitted) % cache.capacity if cache.capacity else 0",
     "cache.head = head"),
    ("the ring does not wrap", None, "cache_update", "s = (head + admitted) % cache.capacity", "s = min(head + admitted, cache.capacity - 1)"),
    ("admission beyond the capacity overwrites this update's own slots", None, "cache_update", "if len(candidates) > room:", "if False:"),
    ("the rows that save least are preferred", None, "cache_update", "(-worth(j), j)", "(worth(j), j)"),
    ("equal estimates go to the higher positions", None, "cache_update", "(-worth(j), j)", "(-worth(j), -j)"),
    ("the admission budget is ignored", None, "cache_update", "min(int(budget), cache.capacity)", "cache.capacity"),
    ("the admission budget may exceed the ring", None, "cache_update", "min(int(budget), cache.capacity)", "int(budget)"),
    ("estimates are compared beyond their saturation point", None, "cache_update", "min(int(saving[j]), SAVING_MAX)", "int(saving[j])"),
    ("the chosen rows are written in order of their estimate", None, "cache_update",
     "    for j in candidates:\n        if j not in chosen:\n            dropped += 1\n            continue\n",
     "    dropped += len(candidates) - len(chosen)\n    for j in sorted(chosen, key=lambda j: (-worth(j), j)) if len(candidates) > room else candidates:\n"),
    ("a cached node counts its whole subtree", None, "access_estimate", "if hit[j]:", "if False:"),
    ("a cached node counts nothing", None, "access_estimate", "out[j] = 1\n", "out[j] = 0\n"),
    ("a node's own row of the layer below is not counted", None, "access_estimate", "total = 1 if below is None else int(below[j])", "total = 0"),
    ("a node's own row counts one read at every layer", None, "access_estimate", "total = 1 if below is None else int(below[j])", "total = 1"),
    ("neighbours count one read each at every layer", None, "access_estimate", "total += 1 if below is None else int(below[col[c]])", "total += 1"),
    ("neighbours are looked up by edge number", None, "access_estimate", "int(below[col[c]])", "int(below[c % len(below)])"),
    ("the estimate does not saturate", None, "access_estimate", "min(total, SAVING_MAX)", "total"),
    ("the estimates of a layer feed its own update one layer off", None, "iteration", "saving=saving.get(l),", "saving=saving.get(l - 1) if l > 1 else saving.get(l),"),
    ("the iteration ignores the budget", None, "iteration", "budget=None if admit_budget is None else admit_budget.get(l))", "budget=None)"),
    ("the wrong row is stored", None, "cache_update", "cache.store(s, h[j])", "cache.store(s, h[admitted])"),
    ("a normal row does not keep its own position live", None, "lookup_prune", "live_src[j] = True", "pass"),
    ("pruned nodes are looked up", None, "lookup_prune", "if not live[j]:\n            continue", "if False:\n            continue"),
    ("rows that are not normal keep their neighbours", None, "lookup_prune", "end[j] = start[j]", "pass"),
    ("neighbours of hit rows stay live", None, "lookup_prune", "if normal[j]:", "if live[j]:"),
    ("hits are listed as normal too", None, "lookup_prune", "        else:\n            normal_pos.append(j)", "        normal_pos.append(j)"),
    ("a feature row cut by the end of the written part still counts as intact", "BidirectionalCache", "feature_rank",
     "lo < w_hi and hi > w_lo", "hi <= w_hi and hi > w_lo"),
    ("a feature row touching the written part from the right counts as lost", "BidirectionalCache", "feature_rank",
     "lo < w_hi and hi > w_lo", "lo <= w_hi and hi > w_lo"),
    ("an empty ring displaces the feature row lying across its first byte", "BidirectionalCache", "feature_rank",
     "ring.used > 0 and lo", "lo"),
    ("only the first ring displaces features", "BidirectionalCache", "feature_rank",
     "for l, ring in self.rings.items():", "for l, ring in list(self.rings.items())[:1]:"),
    ("the written part is measured in feature rows", "BidirectionalCache", "feature_rank",
     "w_lo + ring.used * ring.row_bytes", "w_lo + ring.used * self.feat_row_bytes"),
    ("the hottest row is placed next to the embeddings", "BidirectionalCache", "fill_features",
     "self.rank_of[v] = r", "self.rank_of[v] = len(hot_ids) - 1 - r"),
    ("feature rows are placed from the left end", "BidirectionalCache", "fill_features",
     "self.buf[B - (r + 1) * w:B - r * w] = row_image(rows[r], feat_dtype)", "self.buf[r * w:(r + 1) * w] = row_image(rows[r], feat_dtype)"),
    ("the second ring starts right after the first without alignment", "BidirectionalCache", "__init__",
     "at = -(-at // RING_ALIGN) * RING_ALIGN", "at = at"),
    ("the written part of a ring shrinks back when the header wraps", None, "cache_update",
     "cache.used = cache.capacity if head + admitted >= cache.capacity else max(cache.used, head + admitted)",
     "cache.used = (head + admitted) % cache.capacity"),
    ("the written part stops growing one slot early", None, "cache_update",
     "max(cache.used, head + admitted)", "max(cache.used, head + admitted - 1)"),
    ("rings do not write their rows into the shared buffer", "HistoricalCache", "store",
     "if self.storage is not None:", "if False:"),
    ("bf16 rows are laid down as their low halves", None, "row_image", ">> np.uint32(16)", "& np.uint32(0xFFFF)"),
    ("the hot list is in ascending order of the estimate", None, "hot_order", "(-score[v], v)", "(score[v], v)"),
    ("ties in the hot list go to the larger id", None, "hot_order", "(-score[v], v)", "(-score[v], -v)"),
    ("the loss gradient is not averaged over the batch", None, "softmax_xent_grad", "return p / len(h)", "return p"),
    ("the loss gradient forgets the label term", None, "softmax_xent_grad", "p[np.arange(len(h)), np.asarray(labels)] -= 1.0", "pass"),
    ("row norms are sums of squares", None, "row_norms", "np.sqrt((x * x).sum(axis=1))", "(x * x).sum(axis=1)"),
    ("row norms are 1-norms", None, "row_norms", "np.sqrt((x * x).sum(axis=1))", "np.abs(x).sum(axis=1)"),
    ("the backward pass ignores the ReLU", None, "layer_backward", "if relu:", "if False:"),
    ("the ReLU mask lets zeros through", None, "layer_backward", "np.asarray(h_out)[rows] > 0)", "np.asarray(h_out)[rows] >= 0)"),
    ("the backward pass masks the last layer too", None, "backward", "relu=(l < L))", "relu=True)"),
    ("self and neighbour halves of the input gradient are swapped", None, "layer_backward",
     "dsrc[r] += dx[k, :d_in]", "dsrc[r] += dx[k, d_in:]"),
    ("the neighbours' share is not divided by the degree", None, "layer_backward", "dx[k, d_in:] / float(len(nb))", "dx[k, d_in:]"),
    ("the neighbours' share is divided by degree + 1", None, "layer_backward", "/ float(len(nb)))", "/ float(len(nb) + 1))"),
    ("a row's own previous embedding receives no gradient", None, "layer_backward", "dsrc[r] += dx[k, :d_in]", "pass"),
    ("a neighbour sampled by several rows keeps only the last contribution", None, "layer_backward",
     "np.add.at(dsrc, nb, dx[k, d_in:] / float(len(nb)))", "dsrc[nb] = dx[k, d_in:] / float(len(nb))"),
    ("the weight gradient swaps its panels", None, "layer_backward",
     "np.concatenate([np.asarray(h_self, dtype=np.float64), np.asarray(agg, dtype=np.float64)], axis=1)",
     "np.concatenate([np.asarray(agg, dtype=np.float64), np.asarray(h_self, dtype=np.float64)], axis=1)"),
    ("the bias gradient is a mean", None, "layer_backward", "db = dz.sum(axis=0)", "db = dz.mean(axis=0)"),
    ("the input gradient uses the untransposed weights of the self panel twice", None, "layer_backward", "dx = dz @ W.T",
     "dx = dz @ np.concatenate([W[:d_in], W[:d_in]]).T"),
    ("gradient norms are taken one layer off", None, "backward", "gnorm = {l: row_norms(dH[l])", "gnorm = {l: row_norms(dH[l + 1])"),
    ("the GCN propagation leaves the node itself out", None, "aggregate_gcn", "(h[r].astype(np.float64) + h[nb]", "(0 * h[r].astype(np.float64) + h[nb]"),
    ("the GCN propagation divides by the neighbour count only", None, "aggregate_gcn", "/ float(len(nb) + 1)", "/ float(max(len(nb), 1))"),
    ("the GCN layer drops its bias", None, "linear_gcn", "+ np.asarray(b, dtype=np.float64)", "+ 0 * np.asarray(b, dtype=np.float64)"),
    ("the GCN layer never applies ReLU", None, "linear_gcn", "if relu else z", "if False else z"),
    ("the stabilization period ends one iteration early", None, "iteration", "cache_active = i >= stabilization", "cache_active = i >= stabilization - 1"),
    ("the cache is looked up during the stabilization period", None, "iteration", "    if not cache_active:\n        caches = {}\n", ""),
    ("mixed precision: the mean enters the product unrounded", None, "iteration", "AGG[l] = round_bf16(agg64)", 'AGG[l] = round_to(agg64, "f32")'),
    ("mixed precision: the mean is rounded to fp16 instead of bf16", None, "iteration", "AGG[l] = round_bf16(agg64)",
     'AGG[l] = round_to(agg64, "f16").astype(np.float32)'),
    ("mixed precision: the own rows enter the product as fp16", None, "iteration",
     "h_self = round_bf16(H[l - 1][rows].astype(np.float64))", "h_self = H[l - 1][rows]"),
    ("mixed precision: the weights enter the product unrounded", None, "iteration", "W = round_bf16(W)", "W = W"),
    ("mixed precision: hidden embeddings are stored as fp32", None, "iteration",
     'out_dtype = "f32" if l == L else compute_dtype', 'out_dtype = "f32"'),
    ("mixed precision: the last layer is rounded to bf16 too", None, "iteration",
     'out_dtype = "f32" if l == L else compute_dtype', "out_dtype = compute_dtype"),
    ("mixed precision: hidden embeddings are rounded to fp16", None, "iteration",
     'out_dtype = "f32" if l == L else compute_dtype', 'out_dtype = "f32" if l == L else "f16"'),
    ("mixed precision: the output gradient enters the backward products unrounded", None, "layer_backward",
     "dz = round_bf16(dz).astype(np.float64)", "dz = dz"),
    ("mixed precision: the backward product uses unrounded weights", None, "layer_backward",
     "W = round_bf16(W).astype(np.float64)", "W = W"),
    ("mixed precision: the bias gradient sums the rounded output gradient", None, "layer_backward",
     "    db = dz.sum(axis=0)\n", '    db = (round_bf16(dz).astype(np.float64) if compute_dtype == "bf16" else dz).sum(axis=0)\n'),
    ("mixed precision: the weight gradient takes the own rows as fp16", None, "backward",
     'h_self = round_bf16(h_prev[rows].astype(np.float64)) if compute_dtype == "bf16" else h_prev[rows]', "h_self = h_prev[rows]"),
    ("mixed precision: embedding gradients are carried in fp64 between the layers", None, "backward",
     'dh_l = dH[l].astype(np.float32) if compute_dtype == "bf16" else dH[l]', "dh_l = dH[l]"),
    ("mixed precision: the backward pass ignores the setting", None, "backward", "compute_dtype=compute_dtype)", 'compute_dtype="f32")'),
    ("GCN backward: shares are divided by the neighbour count only", None, "layer_backward_gcn",
     "share = dm[k] / float(len(nb) + 1)", "share = dm[k] / float(max(len(nb), 1))"),
    ("GCN backward: the node itself receives nothing", None, "layer_backward_gcn", "        dsrc[r] += share\n", "        pass\n"),
    ("GCN backward: the node itself receives the undivided gradient", None, "layer_backward_gcn", "        dsrc[r] += share\n", "        dsrc[r] += dm[k]\n"),
    ("GCN backward: no ReLU mask", None, "layer_backward_gcn", "if relu:", "if False:"),
    ("GCN backward: a neighbour sampled by several rows keeps the last share", None, "layer_backward_gcn",
     "np.add.at(dsrc, nb, share)", "dsrc[nb] = share"),
    ("GCN backward: the weight gradient is taken from the output", None, "layer_backward_gcn",
     "dW = np.asarray(agg, dtype=np.float64).T @ dz", "dW = np.asarray(agg, dtype=np.float64).T @ np.asarray(dh, dtype=np.float64)[rows]"),
    ("GCN backward: the bias gradient is a mean", None, "layer_backward_gcn", "db = dz.sum(axis=0)", "db = dz.mean(axis=0)"),
    ("GCN backward: the input gradient uses W instead of its transpose", None, "layer_backward_gcn", "dm = dz @ W.T",
     "dm = dz @ W.T if W.shape[0] != W.shape[1] else dz @ W"),
    ("GCN backward: the GraphSAGE rule is applied", None, "backward", 'if model == "gcn":', "if False:"),
    ("cached feature rows are read at the neighbouring rank", "BidirectionalCache", "load",
     "out[k] = self.buf[B - (r + 1) * w:B - r * w].view(np_dt)", "out[k] = self.buf[B - (r + 2) * w:B - (r + 1) * w].view(np_dt) if r + 2 <= self.n_feat else 0"),
]


def _plant(owner, name, old, new):
    target = getattr(O, owner) if owner else O
    original = getattr(target, name)
    src = textwrap.dedent(inspect.getsource(original))
    assert src.count(old) == 1, f"the text to change occurs {src.count(old)} times in {name}"
    scope = {}
    exec(compile(src.replace(old, new), f"<mutant of {name}>", "exec"), O.__dict__, scope)
    setattr(target, name, scope[name])
    return target, name, original


def _first_failing_pin():
    for fn, cases in PINS:
        for args in cases:
            try:
                fn(*args)
            except Exception as e:  # an assertion of the pin, or the mistake making the oracle itself stumble
                return f"{fn.__name__}{args}: {type(e).__name__}"
    return None


def test_pins_pass_on_the_unmodified_oracle():
    assert _first_failing_pin() is None


@pytest.mark.parametrize("what,owner,name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(what, owner, name, old, new):
    target, attr, original = _plant(owner, name, old, new)
    try:
        caught = _first_failing_pin()
    finally:
        setattr(target, attr, original)
    assert caught is not None, f"no pin notices that {what}"
