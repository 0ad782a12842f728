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
#include <atomic>

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

// Slot holding a usable embedding of node v at iteration cv.iter, or -1.
__device__ __forceinline__ int32_t cache_lookup(const CacheView& cv, int32_t v) {
    if (v < 0 || v >= cv.num_nodes) return -1;
    const int32_t s = cv.map[v];
    if (s < 0 || s >= cv.capacity || cv.slot_node[s] != v) return -1;
    const int64_t age = cv.iter - (int64_t)cv.slot_stamp[s];
    return (age >= 1 && age <= (int64_t)cv.t_stale) ? s : -1;
}

// One chunk of FG_SCAN_BLOCK positions, executed by a whole workgroup of FG_SCAN_BLOCK threads.
__device__ __forceinline__ void classify_mark_chunk(
    const CacheView& cv, int has_cache, const int32_t* __restrict__ ids, int n, const uint8_t* __restrict__ live,
    const int32_t* __restrict__ row_start, int32_t* __restrict__ row_end, const int32_t* __restrict__ col, int64_t nnz,
    int n_src, uint8_t* __restrict__ live_src, uint8_t* __restrict__ hit_out, uint8_t* __restrict__ cls_ws,
    int32_t* __restrict__ slot_ws, int32_t* __restrict__ blk_counts, int chunk, bool have_candidates = false) {
    const int j = chunk * FG_SCAN_BLOCK + threadIdx.x;
    const bool in = j < n;
    // everything this position may need is requested at once (one memory round trip instead of a chain of four)
    const uint8_t live_j = in ? (live ? live[j] : (uint8_t)1) : (uint8_t)0;
    int32_t s0 = 0, e0 = 0, slot_j = -1, id_j = -1;
    if (in && row_start) {
        s0 = row_start[j];
        e0 = row_end[j];
    }
    if (in && has_cache) {
        if (have_candidates) slot_j = slot_ws[j];  // the node's usable slot or -1, looked up for every position beforehand
        else id_j = ids[j];
    }
    const bool is_live = live_j != 0;
    bool hit = false;
    int32_t slot = -1;
    if (is_live && has_cache) {
        slot = have_candidates ? slot_j : cache_lookup(cv, id_j);
        hit = slot >= 0;
    }
    const bool normal = is_live && !hit;
    if (in) {
        cls_ws[j] = is_live ? (hit ? CLS_HIT : CLS_NORMAL) : CLS_DEAD;
        slot_ws[j] = slot;
        if (hit_out) hit_out[j] = hit ? 1 : 0;
        if (row_start) {
            if (!normal) {
                row_end[j] = s0;
            } else {
                if (live_src && j < n_src) live_src[j] = 1;
                if (live_src && s0 >= 0 && s0 <= e0 && (int64_t)e0 <= nnz) {
                    // neighbour positions eight at a time: the loads go out together (a slot past the end re-reads
                    // the last one), then the marks (many writers, one value)
                    for (int32_t e = s0; e < e0; e += 8) {
                        int32_t c[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) c[u] = col[e + u < e0 ? e + u : e0 - 1];
#pragma unroll
                        for (int u = 0; u < 8; ++u)
                            if (e + u < e0 && c[u] >= 0 && c[u] < n_src) live_src[c[u]] = 1;
                    }
                }
            }
        }
    }
    const int c_live = __syncthreads_count(is_live);
    const int c_hit = __syncthreads_count(hit);
    if (threadIdx.x == 0) {
        blk_counts[3 * chunk + 0] = c_live;
        blk_counts[3 * chunk + 1] = c_hit;
        blk_counts[3 * chunk + 2] = c_live - c_hit;
    }
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void classify_mark_kernel(
    CacheView cv, int has_cache, const int32_t* __restrict__ ids, int n, const uint8_t* __restrict__ live,
    const int32_t* __restrict__ row_start, int32_t* __restrict__ row_end, const int32_t* __restrict__ col, int64_t nnz,
    int n_src, uint8_t* __restrict__ live_src, uint8_t* __restrict__ hit_out, uint8_t* __restrict__ cls_ws,
    int32_t* __restrict__ slot_ws, int32_t* __restrict__ blk_counts) {
    classify_mark_chunk(cv, has_cache, ids, n, live, row_start, row_end, col, nnz, n_src, live_src, hit_out, cls_ws, slot_ws,
                        blk_counts, blockIdx.x);
}

__device__ __forceinline__ void compact_lists_chunk(
    const int32_t* __restrict__ ids, int n, const uint8_t* __restrict__ cls_ws, const int32_t* __restrict__ slot_ws,
    const int32_t* __restrict__ blk_counts, int32_t* __restrict__ hit_pos, int32_t* __restrict__ hit_slot,
    int32_t* __restrict__ normal_pos, int32_t* __restrict__ normal_ids, int64_t* __restrict__ counts_out, int chunk,
    int n_chunks, long long* red, int* sc) {
    // this position's class, slot and id are requested before the counts of the preceding workgroups are added up
    const int j = chunk * FG_SCAN_BLOCK + threadIdx.x;
    const uint8_t c = j < n ? cls_ws[j] : CLS_DEAD;
    const int32_t slot_j = j < n ? slot_ws[j] : -1;
    const int32_t id_j = (j < n && normal_ids) ? ids[j] : -1;
    long long p_live = 0, p_hit = 0, p_norm = 0;
    for (int b = threadIdx.x; b < chunk; b += FG_SCAN_BLOCK) {
        p_live += blk_counts[3 * b + 0];
        p_hit += blk_counts[3 * b + 1];
        p_norm += blk_counts[3 * b + 2];
    }
    p_live = fg_block_sum(p_live, red);
    p_hit = fg_block_sum(p_hit, red);
    p_norm = fg_block_sum(p_norm, red);

    int t_hit, t_norm;
    const int r_hit = fg_block_rank(c == CLS_HIT, t_hit, sc);
    const int r_norm = fg_block_rank(c == CLS_NORMAL, t_norm, sc);
    if (c == CLS_HIT && hit_pos) {
        hit_pos[p_hit + r_hit] = j;
        hit_slot[p_hit + r_hit] = slot_j;
    }
    if (c == CLS_NORMAL) {
        normal_pos[p_norm + r_norm] = j;
        if (normal_ids) normal_ids[p_norm + r_norm] = id_j;
    }
    if (chunk == n_chunks - 1 && threadIdx.x == 0) {
        counts_out[0] = p_live + t_hit + t_norm;
        counts_out[1] = p_hit + t_hit;
        counts_out[2] = p_norm + t_norm;
    }
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void compact_lists_kernel(
    const int32_t* __restrict__ ids, int n, const uint8_t* __restrict__ cls_ws, const int32_t* __restrict__ slot_ws,
    const int32_t* __restrict__ blk_counts, int32_t* __restrict__ hit_pos, int32_t* __restrict__ hit_slot,
    int32_t* __restrict__ normal_pos, int32_t* __restrict__ normal_ids, int64_t* __restrict__ counts_out) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    compact_lists_chunk(ids, n, cls_ws, slot_ws, blk_counts, hit_pos, hit_slot, normal_pos, normal_ids, counts_out, blockIdx.x,
                        gridDim.x, red, sc);
}

// ---- the whole top-down pass with short dependency chains ---------------------------------------------------
//
// Layer by layer, every step is a chain of dependent random reads (liveness -> id -> map -> slot owner and stamp
// -> row range -> neighbour positions): latency, not bandwidth or launch overhead, sets its time. The cache
// lookups do not depend on liveness, so one preparation launch does them for every position of every cached
// layer at once (and clears the liveness arrays); the per-layer phases that follow only combine flags and walk
// the rows. The compaction of a layer shares a launch with the classification of the layer below.
constexpr int TD_MAX_LAYERS = 8;

struct TdLayer {
    CacheView cv;
    int has_cache;
    const int32_t* ids;
    int n;
    const uint8_t* live;
    const int32_t* row_start;
    int32_t* row_end;
    const int32_t* col;
    int64_t nnz;
    int n_src;
    uint8_t* live_src;
    uint8_t* hit;
    int32_t* hit_pos;
    int32_t* hit_slot;
    int32_t* normal_pos;
    int32_t* normal_ids;
    int64_t* counts;
    uint8_t* cls;
    int32_t* slot;
    int32_t* blk;
};

struct TdArgs {
    TdLayer layer[TD_MAX_LAYERS];
    int count;
};

__global__ __launch_bounds__(256) void td_prepare_kernel(TdArgs a) {
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    for (int i = 0; i < a.count; ++i) {
        const TdLayer& L = a.layer[i];
        if (L.has_cache)
            for (int64_t j = gtid; j < L.n; j += gsize) L.slot[j] = cache_lookup(L.cv, L.ids[j]);
        uint8_t* p = L.live_src;
        if (!p) continue;
        const int64_t n = L.n_src;
        const int64_t head = ((uintptr_t)p & 3) ? 4 - (int64_t)((uintptr_t)p & 3) : 0;  // bytes up to 4-byte alignment
        const int64_t words = n > head ? (n - head) >> 2 : 0;
        for (int64_t q = gtid; q < words; q += gsize) ((uint32_t*)(p + head))[q] = 0u;
        for (int64_t q = gtid; q < head && q < n; q += gsize) p[q] = 0;
        for (int64_t q = head + 4 * words + gtid; q < n; q += gsize) p[q] = 0;
    }
}

// workgroups [0, nc_cur) classify layer `cur`; workgroups [nc_cur, nc_cur + nc_prev) compact layer `prev`
__global__ __launch_bounds__(FG_SCAN_BLOCK) void td_phase_kernel(TdArgs a, int cur, int prev, int nc_cur, int nc_prev) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    const int b = blockIdx.x;
    if (b < nc_cur) {
        const TdLayer& L = a.layer[cur];
        classify_mark_chunk(L.cv, L.has_cache, L.ids, L.n, L.live, L.row_start, L.row_end, L.col, L.nnz, L.n_src, L.live_src,
                            L.hit, L.cls, L.slot, L.blk, b, true);
    } else if (prev >= 0) {
        const TdLayer& P = a.layer[prev];
        if (nc_prev == 0) {
            if (threadIdx.x < 3) P.counts[threadIdx.x] = 0;
        } else {
            compact_lists_chunk(P.ids, P.n, P.cls, P.slot, P.blk, P.has_cache ? P.hit_pos : nullptr, P.hit_slot, P.normal_pos,
                                P.normal_ids, P.counts, b - nc_cur, nc_prev, red, sc);
        }
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

static fg_status_t lookup_prune_launch(const fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev,
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
        cv = CacheView{ly.map, ly.slot_node, ly.slot_stamp, ly.capacity, cache->num_nodes, iter, fg_t_stale_at(cache, iter)};
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

extern "C" fg_status_t fg_lookup_prune(const fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev,
                                       int32_t n, const uint8_t* live_dev, const int32_t* row_start_dev,
                                       int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz, int32_t n_src,
                                       uint8_t* live_src_dev, uint8_t* hit_dev, int32_t* hit_pos_dev,
                                       int32_t* hit_slot_dev, int32_t* normal_pos_dev, int32_t* normal_ids_dev,
                                       int64_t* counts_dev, void* ws_dev, size_t ws_bytes, void* stream) {
    return lookup_prune_launch(cache, layer, iter, ids_dev, n, live_dev, row_start_dev, row_end_dev, col_dev, nnz, n_src,
                               live_src_dev, hit_dev, hit_pos_dev, hit_slot_dev, normal_pos_dev, normal_ids_dev, counts_dev,
                               ws_dev, ws_bytes, stream);
}

// ---- the same call for callers that cannot allocate: its scratch memory is a device array of the library -------------
//
// classify_mark_kernel leaves a class and a slot per position and three counts per workgroup there, compact_lists_kernel
// reads them back: everything read has been written by the same call, so nothing needs clearing between calls.
constexpr int64_t LP_STATIC_MAX_N = FG_LOOKUP_PRUNE_STATIC_MAX_N;
constexpr size_t LP_STATIC_BYTES = ((size_t)LP_STATIC_MAX_N + 255) / 256 * 256                      // class per position
                                   + ((size_t)LP_STATIC_MAX_N * 4 + 255) / 256 * 256               // slot per position
                                   + (((size_t)LP_STATIC_MAX_N + FG_SCAN_BLOCK - 1) / FG_SCAN_BLOCK * 12 + 255) / 256 * 256;
static __device__ __align__(256) unsigned char scratch[LP_STATIC_BYTES];

constexpr int LP_MAX_DEVICES = 64;
static std::atomic<void*> scratch_of_device[LP_MAX_DEVICES];   // each device holds its own copy of the array

extern "C" fg_status_t fg_lookup_prune_static(const fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev,
                                              int32_t n, const uint8_t* live_dev, const int32_t* row_start_dev,
                                              int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz, int32_t n_src,
                                              uint8_t* live_src_dev, uint8_t* hit_dev, int32_t* hit_pos_dev,
                                              int32_t* hit_slot_dev, int32_t* normal_pos_dev, int32_t* normal_ids_dev,
                                              int64_t* counts_dev, void* stream) {
    if (n > LP_STATIC_MAX_N)
        FG_FAIL(FG_ERR_SHAPE, "fg_lookup_prune_static: n = %d exceeds the %lld positions its built-in scratch memory holds "
                "(use fg_lookup_prune with a workspace)", n, (long long)LP_STATIC_MAX_N);
    if (ws_layout(n > 0 ? n : 0).total > LP_STATIC_BYTES)
        FG_FAIL(FG_ERR_SHAPE, "fg_lookup_prune_static: n = %d needs more scratch memory than is built in", n);
    int device = -1;
    FG_HIP(hipGetDevice(&device));
    if (device < 0 || device >= LP_MAX_DEVICES)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_lookup_prune_static: device %d outside 0..%d", device, LP_MAX_DEVICES - 1);
    void* ws = scratch_of_device[device].load(std::memory_order_acquire);
    if (!ws) {
        // the array's name is not a device address on the host: ask for the address of this device's copy, once
        FG_HIP(hipGetSymbolAddress(&ws, HIP_SYMBOL(scratch)));
        if (!ws) FG_FAIL(FG_ERR_HIP, "fg_lookup_prune_static: the scratch array has no address on device %d", device);
        scratch_of_device[device].store(ws, std::memory_order_release);
    }
    return lookup_prune_launch(cache, layer, iter, ids_dev, n, live_dev, row_start_dev, row_end_dev, col_dev, nnz, n_src,
                               live_src_dev, hit_dev, hit_pos_dev, hit_slot_dev, normal_pos_dev, normal_ids_dev, counts_dev,
                               ws, LP_STATIC_BYTES, stream);
}

extern "C" size_t fg_top_down_workspace_bytes(int32_t n_layers, const fg_top_down_layer_t* layers) {
    if (n_layers <= 0 || !layers) return 0;
    size_t total = 0;
    for (int i = 0; i < n_layers; ++i) total += ws_layout(layers[i].n > 0 ? layers[i].n : 0).total;
    return total;
}

extern "C" fg_status_t fg_top_down(const fg_cache_t* cache, int64_t iter, int32_t n_layers,
                                   const fg_top_down_layer_t* layers, void* ws_dev, size_t ws_bytes, void* stream) {
    if (n_layers <= 0 || n_layers > TD_MAX_LAYERS || !layers)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: n_layers = %d must be in 1..%d and layers non-NULL", n_layers, TD_MAX_LAYERS);
    TdArgs a{};
    a.count = n_layers;
    size_t off = 0;
    for (int i = 0; i < n_layers; ++i) {
        const fg_top_down_layer_t& in = layers[i];
        TdLayer& L = a.layer[i];
        if (in.n < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d].n = %d is negative", i, in.n);
        if (!in.counts_dev) FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d].counts_dev is NULL", i);
        if (in.n > 0 && (!in.ids_dev || !in.normal_pos_dev))
            FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d] needs ids_dev and normal_pos_dev", i);
        const bool has_block = in.row_start_dev || in.row_end_dev;
        if (has_block) {
            if (!in.row_start_dev || !in.row_end_dev || (in.nnz > 0 && !in.col_dev && in.live_src_dev))
                FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d]: a block needs row_start_dev, row_end_dev and col_dev together", i);
            if (in.nnz < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d].nnz is negative", i);
            if (in.live_src_dev && in.n_src < in.n)
                FG_FAIL(FG_ERR_SHAPE, "fg_top_down: layers[%d]: n_src = %d is smaller than n = %d", i, in.n_src, in.n);
        } else if (in.live_src_dev) {
            FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d]: live_src_dev without a block", i);
        }
        if (i + 1 < n_layers && in.live_src_dev && layers[i + 1].live_dev != in.live_src_dev)
            FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d].live_src_dev must be layers[%d].live_dev", i, i + 1);
        L.has_cache = 0;
        if (in.cache_layer != 0) {
            if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d] names cache layer %d but cache is NULL", i, in.cache_layer);
            if (in.cache_layer < 1 || in.cache_layer > cache->n_layers)
                FG_FAIL(FG_ERR_SHAPE, "fg_top_down: layers[%d]: cache layer %d outside 1..%d", i, in.cache_layer, cache->n_layers);
            if (in.n > 0 && (!in.hit_dev || !in.hit_pos_dev || !in.hit_slot_dev))
                FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: layers[%d]: hit_dev, hit_pos_dev and hit_slot_dev are required with a cache", i);
            const fg_layer& ly = cache->layers[in.cache_layer - 1];
            L.cv = CacheView{ly.map, ly.slot_node, ly.slot_stamp, ly.capacity, cache->num_nodes, iter, fg_t_stale_at(cache, iter)};
            L.has_cache = 1;
        }
        const WsLayout w = ws_layout(in.n);
        L.ids = in.ids_dev;
        L.n = in.n;
        L.live = in.live_dev;
        L.row_start = has_block ? in.row_start_dev : nullptr;
        L.row_end = in.row_end_dev;
        L.col = in.col_dev;
        L.nnz = in.nnz;
        L.n_src = in.n_src;
        L.live_src = has_block ? in.live_src_dev : nullptr;
        L.hit = in.hit_dev;
        L.hit_pos = in.hit_pos_dev;
        L.hit_slot = in.hit_slot_dev;
        L.normal_pos = in.normal_pos_dev;
        L.normal_ids = in.normal_ids_dev;
        L.counts = in.counts_dev;
        L.cls = (uint8_t*)((char*)ws_dev + off + w.cls);
        L.slot = (int32_t*)((char*)ws_dev + off + w.slot);
        L.blk = (int32_t*)((char*)ws_dev + off + w.blk);
        off += w.total;
    }
    if (!ws_dev || ws_bytes < off) FG_FAIL(FG_ERR_SHAPE, "fg_top_down: workspace of %zu bytes given, %zu needed", ws_bytes, off);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: workspace must be 16-byte aligned");
    fg_clear_error();
    hipStream_t st = (hipStream_t)stream;
    int64_t prep = 0;
    for (int i = 0; i < n_layers; ++i) {
        if (a.layer[i].has_cache) prep = prep > a.layer[i].n ? prep : a.layer[i].n;
        // every liveness array is cleared by this launch, however short it is
        if (a.layer[i].live_src) prep = prep > fg_ceil_div(a.layer[i].n_src, 4) ? prep : fg_ceil_div(a.layer[i].n_src, 4);
    }
    if (prep > 0) {
        const int64_t blocks = fg_ceil_div(prep, 256) < 2048 ? fg_ceil_div(prep, 256) : 2048;
        hipLaunchKernelGGL(td_prepare_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
        FG_LAUNCH_CHECK("td_prepare_kernel");
    }
    for (int i = 0; i <= n_layers; ++i) {
        const int nc_cur = i < n_layers ? (int)fg_ceil_div(a.layer[i].n, FG_SCAN_BLOCK) : 0;
        const int nc_prev = i > 0 ? (int)fg_ceil_div(a.layer[i - 1].n, FG_SCAN_BLOCK) : 0;
        const int grid = nc_cur + (i > 0 ? (nc_prev > 0 ? nc_prev : 1) : 0);
        if (grid == 0) continue;
        hipLaunchKernelGGL(td_phase_kernel, dim3(grid), dim3(FG_SCAN_BLOCK), 0, st, a, i < n_layers ? i : -1, i > 0 ? i - 1 : -1,
                           nc_cur, nc_prev);
        FG_LAUNCH_CHECK("td_phase_kernel");
    }
    return FG_OK;
}
