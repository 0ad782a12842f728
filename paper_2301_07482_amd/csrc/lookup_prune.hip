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
// -> row range -> neighbour positions): latency, not bandwidth or launch overhead, sets its time, and every
// launch boundary adds to it. The pass is therefore cut into as few launches as its data dependences allow:
//
//   1. walk + lookups. The cache lookups do not depend on liveness, so every position of every cached layer is
//      looked up here. Beside them, one wavefront per seed row walks down the first two blocks: a seed that is
//      computed marks itself and its neighbours in the layer below, and each of those (one per lane) that is not
//      cached marks itself and its own neighbours in the layer below that. A node reached from several seeds is
//      walked once per seed; the marks are idempotent, and for sampled mini-batches (few repeats) the extra work
//      is small. This settles the liveness of the two layers below the seeds in one launch instead of two.
//   2. classify: every layer whose liveness is known (up to three) at once: liveness, hit or normal, row cut,
//      per-workgroup counts; the lowest of them marks the layer below it.
//   3. compact those layers (ballot ranks + the counts of the preceding workgroups), in the same launch as the
//      classification of the next layer down, and so on until the last layer is compacted.
//
// Liveness travels between launches as one byte per position in the workspace ("marks"), which are all zero between
// calls: whoever reads a mark clears it. The byte arrays the caller gets (live_src) are written in full by the
// classification of their layer, so nothing has to be cleared ahead of the marking.
constexpr int TD_MAX_LAYERS = 8;
constexpr int TD_WALK_THREADS = 256;
constexpr uint32_t TD_PUBLISHED = 0x80000000u;   // a chunk's counts as one word: this bit, live count << 12, hit count
constexpr int TD_FUSED_MAX_BLOCKS = 256;         // workgroups of a launch whose chunks wait for each other: all resident at once
constexpr int TD_SPIN_LIMIT = 1 << 20;           // polls of a predecessor's word before a chunk gives up (never reached)

struct TdLayer {
    CacheView cv;
    int has_cache;
    const int32_t* ids;
    int n;                 // positions of the layer: the caller's bound (every array holds this many) ...
    const int64_t* n_dev;  // ... and, if non-null, the count in device memory: positions at or beyond it are dead
    const uint8_t* live;   // liveness given by the caller (seed layer, or a layer whose upper neighbour marks nothing); may be null = all live
    uint8_t* mark;         // workspace, one byte per position, zero between calls: set by the layer above (or the walk)
    uint8_t* live_out;     // non-null: liveness = mark, written here in full (the caller's live_src array of the layer above)
    const int32_t* row_start;
    int32_t* row_end;
    const int32_t* col;
    int64_t nnz;
    int n_src;
    uint8_t* mark_below;   // where normal rows mark the layer below: the next layer's `mark`, or the caller's live_src bytes
                           // (last layer of the list; cleared by the first launch), or null
    int n_mark;            // positions of the layer below that can be marked
    uint8_t* clear_below;  // non-null: mark_below is the caller's array and is cleared by the first launch
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

__device__ __forceinline__ int td_chunks(int n) { return (n + FG_SCAN_BLOCK - 1) / FG_SCAN_BLOCK; }

// positions of the layer that exist: the device-side count where the caller gave one, never above the bound
__device__ __forceinline__ int td_count(const TdLayer& L) {
    if (!L.n_dev) return L.n;
    const int64_t c = *L.n_dev;
    return c < 0 ? 0 : (c < (int64_t)L.n ? (int)c : L.n);
}

// Marks the neighbours of one row, eight loads in flight (a slot past the end re-reads the last one).
__device__ __forceinline__ void td_mark_row(const int32_t* __restrict__ col, int32_t s, int32_t e, uint8_t* __restrict__ mark,
                                            int n_mark) {
    for (int32_t x = s; x < e; x += 8) {
        int32_t c[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) c[u] = col[x + u < e ? x + u : e - 1];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (x + u < e && c[u] >= 0 && c[u] < n_mark) mark[c[u]] = 1;
    }
}

// One wavefront per seed row; lane k takes the row itself (k = 0) or its k-th neighbour and, with two hops, walks that
// node's row of the next block.
__device__ __forceinline__ void td_walk_rows(const TdArgs& a, int hops, int block, int n_blocks) {
    const TdLayer& A = a.layer[0];
    const TdLayer& B = a.layer[1];
    const int lane = threadIdx.x & 63;
    const int n_waves = n_blocks * (TD_WALK_THREADS / 64);
    const int n_seed = td_count(A);
    for (int r = (block * TD_WALK_THREADS + (int)threadIdx.x) >> 6; r < n_seed; r += n_waves) {
        const uint8_t live_r = A.live ? A.live[r] : (uint8_t)1;
        const int32_t s0 = A.row_start[r], e0 = A.row_end[r];
        const int32_t id_r = A.has_cache ? A.ids[r] : -1;
        if (!live_r) continue;
        if (A.has_cache && cache_lookup(A.cv, id_r) >= 0) continue;   // a cached seed needs nothing below it
        const int deg = (s0 >= 0 && s0 <= e0 && (int64_t)e0 <= A.nnz) ? e0 - s0 : 0;
        for (int k = lane; k <= deg; k += 64) {
            const int32_t t = k == 0 ? r : A.col[s0 + k - 1];
            if (t < 0 || t >= A.n_mark) continue;
            if (hops < 2) {
                A.mark_below[t] = 1;
                continue;
            }
            // everything this node may need is requested before anything is stored
            const int32_t id_t = B.has_cache ? B.ids[t] : -1;
            const int32_t s1 = B.row_start[t], e1 = B.row_end[t];
            const bool cached = B.has_cache && cache_lookup(B.cv, id_t) >= 0;
            A.mark_below[t] = 1;
            if (cached || !B.mark_below) continue;
            if (t < B.n_mark) B.mark_below[t] = 1;
            if (s1 >= 0 && s1 <= e1 && (int64_t)e1 <= B.nnz) td_mark_row(B.col, s1, e1, B.mark_below, B.n_mark);
        }
    }
}

// Launch 1: workgroups [0, walk_blocks) walk down from the seeds; the others look every position of every cached layer up
// and clear the caller's liveness array below the last layer, if that is wanted.
__global__ __launch_bounds__(TD_WALK_THREADS) void td_walk_kernel(TdArgs a, int hops, int walk_blocks, int clear_published) {
    if ((int)blockIdx.x < walk_blocks) {
        td_walk_rows(a, hops, blockIdx.x, walk_blocks);
        return;
    }
    const int64_t gtid = (int64_t)(blockIdx.x - walk_blocks) * blockDim.x + threadIdx.x;
    const int64_t gsize = (int64_t)(gridDim.x - walk_blocks) * blockDim.x;
    for (int i = 0; i < a.count; ++i) {
        const TdLayer& L = a.layer[i];
        if (L.has_cache) {
            const int n_i = td_count(L);
            for (int64_t j = gtid; j < n_i; j += gsize) L.slot[j] = cache_lookup(L.cv, L.ids[j]);
        }
        if (clear_published)      // the words the chunks of the fused launches publish their counts in
            for (int64_t q = gtid; q < td_chunks(L.n); q += gsize) L.blk[3 * q] = 0;
        uint8_t* p = L.clear_below;
        if (!p) continue;
        const int64_t n = L.n_src;
        const int64_t head = ((uintptr_t)p & 3) ? 4 - (int64_t)((uintptr_t)p & 3) : 0;  // bytes up to 4-byte alignment
        const int64_t words = n > head ? (n - head) >> 2 : 0;
        for (int64_t q = gtid; q < words; q += gsize) ((uint32_t*)(p + head))[q] = 0u;
        for (int64_t q = gtid; q < head && q < n; q += gsize) p[q] = 0;
        for (int64_t q = head + 4 * words + gtid; q < n; q += gsize) p[q] = 0;
    }
}

// One chunk of FG_SCAN_BLOCK positions of one layer: liveness (from the caller or from the marks, which are cleared),
// class, row cut, and, if `mark`, the marks of a normal row in the layer below. The class and slot of this thread's position
// are returned; `publish`: the chunk's counts go out as one word (see td_fused_kernel) instead of three.
__device__ __forceinline__ void td_classify_chunk(const TdLayer& L, int chunk, bool mark, bool publish, uint8_t& cls_out,
                                                  int32_t& slot_out, int& live_out, int& hit_out) {
    const int j = chunk * FG_SCAN_BLOCK + threadIdx.x;
    const bool in = j < L.n;                // within the arrays: flags and class are written
    const bool there = j < td_count(L);     // a position of this mini-batch
    uint8_t live_j = 0;
    if (in) live_j = L.live_out ? L.mark[j] : ((there && L.live) ? L.live[j] : (uint8_t)1);
    int32_t s0 = 0, e0 = 0, slot_j = -1;
    if (there && L.row_start) {
        s0 = L.row_start[j];
        e0 = L.row_end[j];
    }
    if (there && L.has_cache) slot_j = L.slot[j];   // the node's usable slot or -1, looked up for every position by launch 1
    const bool marked = live_j != 0;        // (a mark beyond the count can only come from a column out of range: cleared, ignored)
    const bool is_live = marked && there;
    const bool hit = is_live && L.has_cache && slot_j >= 0;
    const int32_t slot = hit ? slot_j : -1;
    const bool normal = is_live && !hit;
    cls_out = is_live ? (hit ? CLS_HIT : CLS_NORMAL) : CLS_DEAD;
    slot_out = slot;
    if (in) {
        if (L.live_out) {
            L.live_out[j] = is_live ? 1 : 0;
            if (marked) L.mark[j] = 0;
        }
        if (!publish) {
            L.cls[j] = cls_out;
            L.slot[j] = slot;
        }
        if (L.hit) L.hit[j] = hit ? 1 : 0;
        if (L.row_start && there) {
            if (!normal) {
                L.row_end[j] = s0;
            } else if (mark && L.mark_below) {
                if (j < L.n_mark) L.mark_below[j] = 1;
                if (s0 >= 0 && s0 <= e0 && (int64_t)e0 <= L.nnz) td_mark_row(L.col, s0, e0, L.mark_below, L.n_mark);
            }
        }
    }
    const int c_live = __syncthreads_count(is_live);
    const int c_hit = __syncthreads_count(hit);
    live_out = c_live;
    hit_out = c_hit;
    if (threadIdx.x == 0) {
        if (publish) {
            __hip_atomic_store((uint32_t*)&L.blk[3 * chunk], TD_PUBLISHED | ((uint32_t)c_live << 12) | (uint32_t)c_hit, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        } else {
            L.blk[3 * chunk + 0] = c_live;
            L.blk[3 * chunk + 1] = c_hit;
            L.blk[3 * chunk + 2] = c_live - c_hit;
        }
    }
}

struct TdPhase {
    int cls_first, cls_last;   // layers classified by this launch (cls_first > cls_last: none)
    int mark_from;             // those at or beyond this index also mark the layer below
    int cmp_first, cmp_last;   // layers compacted by this launch
    int cls_blocks;            // workgroups that classify; the rest compact
};

__global__ __launch_bounds__(FG_SCAN_BLOCK) void td_phase_kernel(TdArgs a, TdPhase p) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    int b = blockIdx.x;
    if (b < p.cls_blocks) {
        for (int i = p.cls_first; i <= p.cls_last; ++i) {
            const int nc = td_chunks(a.layer[i].n);
            if (b < nc) {
                uint8_t c;
                int32_t slot;
                int c_live, c_hit;
                td_classify_chunk(a.layer[i], b, i >= p.mark_from, false, c, slot, c_live, c_hit);
                return;
            }
            b -= nc;
        }
        return;
    }
    b -= p.cls_blocks;
    for (int i = p.cmp_first; i <= p.cmp_last; ++i) {
        const TdLayer& P = a.layer[i];
        const int nc = td_chunks(P.n);
        if (nc == 0) {      // an empty layer has one workgroup, which writes its counts
            if (b == 0) {
                if (threadIdx.x < 3) P.counts[threadIdx.x] = 0;
                return;
            }
            b -= 1;
            continue;
        }
        if (b < nc) {
            compact_lists_chunk(P.ids, P.n, P.cls, P.slot, P.blk, P.has_cache ? P.hit_pos : nullptr, P.hit_slot, P.normal_pos,
                                P.normal_ids, P.counts, b, nc, red, sc);
            return;
        }
        b -= nc;
    }
}

// Classification and compaction of a group of layers in one launch. A chunk's lists start where those of the chunks before
// it end, so a chunk publishes its counts as one word (zero before the launch: cleared by launch 1) and then polls the words
// of its predecessors in the same layer. The launch is small enough for all of its workgroups to be resident at once
// (the host checks), a chunk waits only for chunks with a smaller index, and the poll is bounded anyway.
__global__ __launch_bounds__(FG_SCAN_BLOCK) void td_fused_kernel(TdArgs a, TdPhase p) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    int b = blockIdx.x;
    for (int i = p.cls_first; i <= p.cls_last; ++i) {
        const TdLayer& L = a.layer[i];
        const int nc = td_chunks(L.n);
        if (nc == 0) {      // an empty layer has one workgroup, which writes its counts
            if (b == 0) {
                if (threadIdx.x < 3) L.counts[threadIdx.x] = 0;
                return;
            }
            b -= 1;
            continue;
        }
        if (b >= nc) {
            b -= nc;
            continue;
        }
        const int j = b * FG_SCAN_BLOCK + threadIdx.x;
        const int32_t id_j = (j < L.n && L.normal_ids) ? L.ids[j] : -1;
        uint8_t c;
        int32_t slot_j;
        int c_live, c_hit;
        td_classify_chunk(L, b, i >= p.mark_from, true, c, slot_j, c_live, c_hit);
        long long p_live = 0, p_hit = 0;
        bool lost = false;
        for (int q = threadIdx.x; q < b; q += FG_SCAN_BLOCK) {
            uint32_t w = 0;
            int polls = 0;
            do {
                w = __hip_atomic_load((const uint32_t*)&L.blk[3 * q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (w & TD_PUBLISHED) break;
                __builtin_amdgcn_s_sleep(2);
            } while (++polls < TD_SPIN_LIMIT);
            lost = lost || !(w & TD_PUBLISHED);
            p_live += (w >> 12) & 0xFFFu;
            p_hit += w & 0xFFFu;
        }
        p_live = fg_block_sum(p_live, red);
        p_hit = fg_block_sum(p_hit, red);
        const long long p_norm = p_live - p_hit;
        const bool any_lost = __syncthreads_or(lost ? 1 : 0) != 0;
        int t_hit, t_norm;
        const int r_hit = fg_block_rank(c == CLS_HIT, t_hit, sc);
        const int r_norm = fg_block_rank(c == CLS_NORMAL, t_norm, sc);
        if (!any_lost) {
            if (c == CLS_HIT && L.has_cache) {
                L.hit_pos[p_hit + r_hit] = j;
                L.hit_slot[p_hit + r_hit] = slot_j;
            }
            if (c == CLS_NORMAL) {
                L.normal_pos[p_norm + r_norm] = j;
                if (L.normal_ids) L.normal_ids[p_norm + r_norm] = id_j;
            }
        }
        if (b == nc - 1 && threadIdx.x == 0) {
            L.counts[0] = any_lost ? -1 : p_live + t_hit + t_norm;
            L.counts[1] = any_lost ? -1 : p_hit + t_hit;
            L.counts[2] = any_lost ? -1 : p_norm + t_norm;
        }
        return;
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

// Workspace of the whole pass: its first half holds class, slot and counts of every layer (laid out back to back for the
// sizes of the call), its second half the marks. The halves never overlap for any sizes that fit, so the marks stay
// all-zero between calls whatever the layer sizes of the calls are.
static size_t td_other_bytes(int32_t n_layers, const fg_top_down_layer_t* layers) {
    size_t total = 0;
    for (int i = 0; i < n_layers; ++i) total += ws_layout(layers[i].n > 0 ? layers[i].n : 0).total;
    return total;
}

extern "C" size_t fg_top_down_workspace_bytes(int32_t n_layers, const fg_top_down_layer_t* layers) {
    if (n_layers <= 0 || !layers) return 0;
    return 2 * td_other_bytes(n_layers, layers) + 512;
}

extern "C" fg_status_t fg_top_down(const fg_cache_t* cache, int64_t iter, int32_t n_layers,
                                   const fg_top_down_layer_t* layers, void* ws_dev, size_t ws_bytes, void* stream) {
    if (n_layers <= 0 || n_layers > TD_MAX_LAYERS || !layers)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: n_layers = %d must be in 1..%d and layers non-NULL", n_layers, TD_MAX_LAYERS);
    const size_t need = fg_top_down_workspace_bytes(n_layers, layers);
    if (!ws_dev || ws_bytes < need) FG_FAIL(FG_ERR_SHAPE, "fg_top_down: workspace of %zu bytes given, %zu needed", ws_bytes, need);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "fg_top_down: workspace must be 16-byte aligned");
    const size_t marks_at = (ws_bytes / 2 + 255) / 256 * 256;   // depends on the workspace alone, not on the layers of the call
    TdArgs a{};
    a.count = n_layers;
    size_t off = 0, mark_off = marks_at;
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
        L.n_dev = in.n_dev;
        L.live = in.live_dev;
        L.row_start = has_block ? in.row_start_dev : nullptr;
        L.row_end = in.row_end_dev;
        L.col = in.col_dev;
        L.nnz = in.nnz;
        L.n_src = in.n_src;
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
        L.mark = (uint8_t*)ws_dev + mark_off;
        mark_off += fg_align_up((size_t)(in.n > 0 ? in.n : 0), 256);
    }
    if (off > marks_at || mark_off > ws_bytes) FG_FAIL(FG_ERR_SHAPE, "fg_top_down: the workspace is too small for these layers");
    // how liveness reaches each layer, and where each layer marks
    for (int i = 0; i < n_layers; ++i) a.layer[i].live_out = nullptr;
    for (int i = 0; i < n_layers; ++i) {
        TdLayer& L = a.layer[i];
        uint8_t* live_src = L.row_start ? layers[i].live_src_dev : nullptr;
        L.mark_below = L.clear_below = nullptr;
        L.n_mark = 0;
        if (!live_src) continue;
        if (i + 1 < n_layers) {      // the layer below is part of the call: marks in the workspace, bytes written by its classification
            L.mark_below = a.layer[i + 1].mark;
            L.n_mark = L.n_src < a.layer[i + 1].n ? L.n_src : a.layer[i + 1].n;
            a.layer[i + 1].live_out = live_src;
        } else {                     // the caller's array is marked directly and cleared first
            L.mark_below = L.clear_below = live_src;
            L.n_mark = L.n_src;
        }
    }
    fg_clear_error();
    hipStream_t st = (hipStream_t)stream;
    // hops the walk takes from the seeds: a block whose marks go to a layer of this call
    int hops = 0;
    if (fg_tuning(FG_TUNE_TOP_DOWN_WALK) != 0 && n_layers >= 2 && a.layer[0].mark_below && a.layer[0].n > 0) {
        hops = 1;
        const int64_t second = (int64_t)a.layer[0].n + a.layer[0].nnz;   // rows of the second block the walk visits, at most
        if (n_layers >= 3 && a.layer[1].row_start && a.layer[1].mark_below && second <= 262144) hops = 2;
    }
    int64_t prep = 0;
    for (int i = 0; i < n_layers; ++i) {
        if (a.layer[i].has_cache) prep = prep > a.layer[i].n ? prep : a.layer[i].n;
        // the caller's liveness array below the last layer is cleared by this launch, however short it is
        if (a.layer[i].clear_below) prep = prep > fg_ceil_div(a.layer[i].n_src, 4) ? prep : fg_ceil_div(a.layer[i].n_src, 4);
    }
    auto chunks = [&](int i) { return (int)fg_ceil_div(a.layer[i].n, FG_SCAN_BLOCK); };
    // The layers are classified in groups: first every layer the walk settled, then one layer per group. A group whose
    // chunks (an empty layer counts as one) all fit on the chip at once is classified and compacted by one launch.
    const bool fuse = fg_tuning(FG_TUNE_TOP_DOWN_WALK) == 1;
    auto group_blocks = [&](int first, int last) {
        int total = 0;
        for (int i = first; i <= last; ++i) total += chunks(i) > 0 ? chunks(i) : 1;
        return total;
    };
    bool any_fused = false;
    for (int first = 0; first < n_layers;) {
        const int last = first == 0 ? hops : first;
        if (fuse && group_blocks(first, last) <= TD_FUSED_MAX_BLOCKS) any_fused = true;
        first = last + 1;
    }
    if (any_fused)      // the words the chunks publish their counts in are cleared by launch 1
        for (int i = 0; i < n_layers; ++i) prep = prep > chunks(i) ? prep : chunks(i);
    const int walk_blocks = hops > 0 ? (int)fg_ceil_div(a.layer[0].n, TD_WALK_THREADS / 64) : 0;
    int64_t prep_blocks = fg_ceil_div(prep, TD_WALK_THREADS);
    if (prep_blocks > 2048) prep_blocks = 2048;
    if (any_fused && prep_blocks < 1) prep_blocks = 1;
    if (walk_blocks + prep_blocks > 0) {
        hipLaunchKernelGGL(td_walk_kernel, dim3((unsigned)(walk_blocks + prep_blocks)), dim3(TD_WALK_THREADS), 0, st, a, hops, walk_blocks,
                           any_fused ? 1 : 0);
        FG_LAUNCH_CHECK("td_walk_kernel");
    }
    // A group that is not fused is classified by one launch and compacted by the next, beside the classification of the group
    // that follows it.
    int cmp_first = 0, cmp_last = -1;          // classified, not yet compacted
    auto compact_pending_with = [&](int cls_first, int cls_last, int mark_from) -> fg_status_t {
        TdPhase p{};
        p.cls_first = cls_first;
        p.cls_last = cls_last;
        p.mark_from = mark_from;
        p.cmp_first = cmp_first;
        p.cmp_last = cmp_last;
        p.cls_blocks = 0;
        for (int i = cls_first; i <= cls_last; ++i) p.cls_blocks += chunks(i);
        const int cmp_blocks = cmp_first <= cmp_last ? group_blocks(cmp_first, cmp_last) : 0;
        if (p.cls_blocks + cmp_blocks > 0) {
            hipLaunchKernelGGL(td_phase_kernel, dim3((unsigned)(p.cls_blocks + cmp_blocks)), dim3(FG_SCAN_BLOCK), 0, st, a, p);
            FG_LAUNCH_CHECK("td_phase_kernel");
        }
        cmp_first = cls_first;
        cmp_last = cls_last;
        return FG_OK;
    };
    for (int first = 0; first < n_layers;) {
        const int last = first == 0 ? hops : first;
        const int mark_from = first == 0 ? hops : first;      // layers above `hops` were marked from by the walk
        if (fuse && group_blocks(first, last) <= TD_FUSED_MAX_BLOCKS) {
            if (cmp_first <= cmp_last) {      // an earlier group still waits for its compaction
                fg_status_t rc = compact_pending_with(0, -1, 0);
                if (rc != FG_OK) return rc;
                cmp_first = 0, cmp_last = -1;
            }
            TdPhase p{};
            p.cls_first = first;
            p.cls_last = last;
            p.mark_from = mark_from;
            hipLaunchKernelGGL(td_fused_kernel, dim3((unsigned)group_blocks(first, last)), dim3(FG_SCAN_BLOCK), 0, st, a, p);
            FG_LAUNCH_CHECK("td_fused_kernel");
        } else {
            fg_status_t rc = compact_pending_with(first, last, mark_from);
            if (rc != FG_OK) return rc;
        }
        first = last + 1;
    }
    if (cmp_first <= cmp_last) {
        fg_status_t rc = compact_pending_with(0, -1, 0);
        if (rc != FG_OK) return rc;
    }
    return FG_OK;
}
