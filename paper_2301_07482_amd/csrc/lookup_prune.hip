// fg_lookup_prune: one layer of the top-down pass of Algorithm 1 (history index lookup, subgraph removal with
// the two-row-array structure of Section 5, V_normal), plus the ordered lists the later stages consume.
//
// Two launches over the layer, no host synchronisation:
//   1. classify: per position, look the node up through the mapping array (Section 4.2: O(1) per node, no
//      dependency between entries), decide dead / hit / normal, cut the row (end = start) if it is not
//      normal, otherwise mark its own position and its neighbours as live in the layer below; leave one
//      (live, hit, normal) count per workgroup.
//   2. compact: ballot/popcount ranks inside each workgroup, offset by the counts of the workgroups before
//      it, give hit_pos/hit_slot/normal_pos in ascending position order.
#include "common.h"
#include "scan.h"

namespace {

struct CacheView {
    const int32_t* map;
    const int32_t* slot_node;
    const int32_t* slot_stamp;
    int64_t capacity;
    int64_t num_nodes;
    int64_t iter;
    int32_t t_stale;
};

constexpr uint8_t CLS_DEAD = 0, CLS_NORMAL = 1, CLS_HIT = 2;

__global__ __launch_bounds__(FG_SCAN_BLOCK) void classify_mark_kernel(
    CacheView cv, int has_cache, const int32_t* __restrict__ ids, int n, const uint8_t* __restrict__ live,
    const int32_t* __restrict__ row_start, int32_t* __restrict__ row_end, const int32_t* __restrict__ col, int64_t nnz,
    int n_src, uint8_t* __restrict__ live_src, uint8_t* __restrict__ hit_out, uint8_t* __restrict__ cls_ws,
    int32_t* __restrict__ slot_ws, int32_t* __restrict__ blk_counts) {
    const int j = blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    const bool in = j < n;
    const bool is_live = in && (live ? live[j] != 0 : true);
    bool hit = false;
    int32_t slot = -1;
    if (is_live && has_cache) {
        const int32_t v = ids[j];
        if (v >= 0 && v < cv.num_nodes) {
            const int32_t s = cv.map[v];
            if (s >= 0 && s < cv.capacity && cv.slot_node[s] == v) {
                const int64_t age = cv.iter - (int64_t)cv.slot_stamp[s];
                if (age >= 1 && age <= (int64_t)cv.t_stale) {
                    hit = true;
                    slot = s;
                }
            }
        }
    }
    const bool normal = is_live && !hit;
    if (in) {
        cls_ws[j] = is_live ? (hit ? CLS_HIT : CLS_NORMAL) : CLS_DEAD;
        slot_ws[j] = slot;
        if (hit_out) hit_out[j] = hit ? 1 : 0;
        if (row_start) {
            const int32_t s0 = row_start[j];
            if (!normal) {
                row_end[j] = s0;
            } else {
                const int32_t e0 = row_end[j];
                if (live_src && j < n_src) live_src[j] = 1;
                if (live_src && s0 >= 0 && s0 <= e0 && (int64_t)e0 <= nnz) {
                    for (int32_t e = s0; e < e0; ++e) {
                        const int32_t c = col[e];
                        if (c >= 0 && c < n_src) live_src[c] = 1;  // many writers, one value
                    }
                }
            }
        }
    }
    const int c_live = __syncthreads_count(is_live);
    const int c_hit = __syncthreads_count(hit);
    if (threadIdx.x == 0) {
        blk_counts[3 * blockIdx.x + 0] = c_live;
        blk_counts[3 * blockIdx.x + 1] = c_hit;
        blk_counts[3 * blockIdx.x + 2] = c_live - c_hit;
    }
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void compact_lists_kernel(
    const int32_t* __restrict__ ids, int n, const uint8_t* __restrict__ cls_ws, const int32_t* __restrict__ slot_ws,
    const int32_t* __restrict__ blk_counts, int32_t* __restrict__ hit_pos, int32_t* __restrict__ hit_slot,
    int32_t* __restrict__ normal_pos, int32_t* __restrict__ normal_ids, int64_t* __restrict__ counts_out) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    long long p_live = 0, p_hit = 0, p_norm = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += FG_SCAN_BLOCK) {
        p_live += blk_counts[3 * b + 0];
        p_hit += blk_counts[3 * b + 1];
        p_norm += blk_counts[3 * b + 2];
    }
    p_live = fg_block_sum(p_live, red);
    p_hit = fg_block_sum(p_hit, red);
    p_norm = fg_block_sum(p_norm, red);

    const int j = blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    const uint8_t c = j < n ? cls_ws[j] : CLS_DEAD;
    int t_hit, t_norm;
    const int r_hit = fg_block_rank(c == CLS_HIT, t_hit, sc);
    const int r_norm = fg_block_rank(c == CLS_NORMAL, t_norm, sc);
    if (c == CLS_HIT && hit_pos) {
        hit_pos[p_hit + r_hit] = j;
        hit_slot[p_hit + r_hit] = slot_ws[j];
    }
    if (c == CLS_NORMAL) {
        normal_pos[p_norm + r_norm] = j;
        if (normal_ids) normal_ids[p_norm + r_norm] = ids[j];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        counts_out[0] = p_live + t_hit + t_norm;
        counts_out[1] = p_hit + t_hit;
        counts_out[2] = p_norm + t_norm;
    }
}

__global__ void zero_counts_kernel(int64_t* counts) {
    if (threadIdx.x < 3) counts[threadIdx.x] = 0;
}

struct WsLayout {
    size_t cls, slot, blk, total;
};
WsLayout ws_layout(int64_t n) {
    WsLayout w;
    const int64_t nb = fg_ceil_div(n > 0 ? n : 1, FG_SCAN_BLOCK);
    w.cls = 0;
    w.slot = fg_align_up((size_t)n, 256);
    w.blk = w.slot + fg_align_up((size_t)n * 4, 256);
    w.total = w.blk + fg_align_up((size_t)nb * 3 * 4, 256);
    return w;
}

}  // namespace

size_t fg_ws_lookup_prune_bytes(int64_t n) { return ws_layout(n).total; }

extern "C" fg_status_t fg_lookup_prune(const fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev,
                                       int32_t n, const uint8_t* live_dev, const int32_t* row_start_dev,
                                       int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz, int32_t n_src,
                                       uint8_t* live_src_dev, uint8_t* hit_dev, int32_t* hit_pos_dev,
                                       int32_t* hit_slot_dev, int32_t* normal_pos_dev, int32_t* normal_ids_dev,
                                       int64_t* counts_dev, void* ws_dev, size_t ws_bytes, void* stream) {
    if (n < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_lookup_prune: n = %d is negative", n);
    if (!counts_dev) FG_FAIL(FG_ERR_INVALID_ARG, "fg_lookup_prune: counts_dev is NULL");
    if (n > 0 && (!ids_dev || !normal_pos_dev))
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_lookup_prune: ids_dev and normal_pos_dev are required");
    const bool has_block = row_start_dev || row_end_dev || col_dev || live_src_dev;
    if (has_block) {
        if (!row_start_dev || !row_end_dev || (nnz > 0 && !col_dev && live_src_dev))
            FG_FAIL(FG_ERR_INVALID_ARG, "fg_lookup_prune: a block needs row_start_dev, row_end_dev and col_dev together");
        if (nnz < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_lookup_prune: nnz = %lld is negative", (long long)nnz);
        if (n_src < n) FG_FAIL(FG_ERR_SHAPE, "fg_lookup_prune: n_src = %d is smaller than n = %d", n_src, n);
    }
    CacheView cv{};
    if (cache) {
        if (layer < 1 || layer > cache->n_layers)
            FG_FAIL(FG_ERR_SHAPE, "fg_lookup_prune: layer %d outside the cached layers 1..%d", layer, cache->n_layers);
        if (n > 0 && (!hit_dev || !hit_pos_dev || !hit_slot_dev))
            FG_FAIL(FG_ERR_INVALID_ARG, "fg_lookup_prune: hit_dev, hit_pos_dev and hit_slot_dev are required with a cache");
        const fg_layer& ly = cache->layers[layer - 1];
        cv = CacheView{ly.map, ly.slot_node, ly.slot_stamp, ly.capacity, cache->num_nodes, iter, cache->t_stale};
    }
    const WsLayout w = ws_layout(n);
    if (n > 0 && (!ws_dev || ws_bytes < w.total))
        FG_FAIL(FG_ERR_SHAPE, "fg_lookup_prune: workspace of %zu bytes given, %zu needed", ws_bytes, w.total);
    if (ws_dev && ((uintptr_t)ws_dev & 15)) FG_FAIL(FG_ERR_INVALID_ARG, "fg_lookup_prune: workspace must be 16-byte aligned");
    fg_clear_error();
    hipStream_t st = (hipStream_t)stream;
    if (has_block && live_src_dev && n_src > 0) {
        fg_status_t rc = fg_launch_fill_u8(live_src_dev, n_src, 0, st);
        if (rc != FG_OK) return rc;
    }
    if (n == 0) {
        hipLaunchKernelGGL(zero_counts_kernel, dim3(1), dim3(64), 0, st, counts_dev);
        FG_LAUNCH_CHECK("zero_counts_kernel");
        return FG_OK;
    }
    char* ws = (char*)ws_dev;
    uint8_t* cls = (uint8_t*)(ws + w.cls);
    int32_t* slot = (int32_t*)(ws + w.slot);
    int32_t* blk = (int32_t*)(ws + w.blk);
    const int nb = (int)fg_ceil_div(n, FG_SCAN_BLOCK);
    hipLaunchKernelGGL(classify_mark_kernel, dim3(nb), dim3(FG_SCAN_BLOCK), 0, st, cv, cache ? 1 : 0, ids_dev, n,
                       live_dev, has_block ? row_start_dev : nullptr, row_end_dev, col_dev, nnz, n_src, live_src_dev,
                       hit_dev, cls, slot, blk);
    FG_LAUNCH_CHECK("classify_mark_kernel");
    hipLaunchKernelGGL(compact_lists_kernel, dim3(nb), dim3(FG_SCAN_BLOCK), 0, st, ids_dev, n, cls, slot, blk,
                       cache ? hit_pos_dev : nullptr, hit_slot_dev, normal_pos_dev, normal_ids_dev, counts_dev);
    FG_LAUNCH_CHECK("compact_lists_kernel");
    return FG_OK;
}
