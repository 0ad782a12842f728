// The historical embedding cache (Section 4.2, embedding side) and its Update (Algorithm 1, last loop;
// admission and check-out by gradient norm, Section 4.1.1; staleness bound, Section 4.1.2).
//
// State per cached layer, all in HBM: map[num_nodes] (slot of a node or -1), table[capacity x dim],
// slot_node[capacity], slot_stamp[capacity], head. A node v is usable at iteration i iff
//   s = map[v] >= 0, slot_node[s] == v and 1 <= i - slot_stamp[s] <= t_stale.
// The back-pointer test makes every location single-writer during an update: admitting into a slot never
// touches the previous owner's map entry, a check-out only writes the node's own map entry, and the slots
// handed out in one update are distinct. The result is therefore the same as the sequential procedure.
//
// Update = 4 launches, no host synchronisation:
//   1. select_tau    one workgroup: m = live count, k = floor(p_grad*m), radix select (11+11+10 bits on the
//                    order-preserving integer image of the fp32 norms) of the norm with rank k; up to 65536
//                    elements are held in registers after one round of loads, longer lists are streamed per pass
//   2. classify      check out hits that are not below tau; flag admissible normal nodes; count per workgroup
//   3. assign_slots  rank admissible nodes in position order (ballot ranks + preceding workgroups' counts),
//                    hand out ring slots head + rank, write slot_node / slot_stamp / map, list (position, slot);
//                    the last workgroup leaves the advanced header in the spare header cell
//   4. row copy      table[slot] = h[position] (the gather kernel)
#include "common.h"
#include "scan.h"

namespace {

struct UpdHeader {        // lives at the start of the update workspace
    uint32_t tau_key;     // order-preserving key of tau
    int32_t mode;         // 0: nothing is below tau, 1: compare with tau_key, 2: everything is below tau
    int64_t n_admit;      // rows to copy (<= capacity)
    int64_t m_live;
};

__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Exact rank-k selection by one workgroup: three radix passes (11, 11 and 10 bits, most significant first)
// over the order-preserving keys. A pass builds a histogram of the keys that match the digits found so far
// with LDS atomics and finds the bin that contains the wanted rank with a workgroup scan. The first two passes
// stream the norms from memory (a few hundred KB, L2-resident after the first); the keys that survive the
// first digit are parked in LDS for the last pass (if they do not fit, the last pass streams as well).
constexpr int SEL_THREADS = 1024;
constexpr int SEL_BINS = 2048;
constexpr int SEL_BPT = SEL_BINS / SEL_THREADS;  // bins owned by a thread in the scan
constexpr int SEL_PARK = 8192;                   // survivors kept in LDS

// Finds the bin holding rank *s_rank in hist[] (counts), stores it in *s_bin and rebases *s_rank to that bin.
__device__ __forceinline__ void select_bin(const unsigned int* hist, long long* red, uint32_t* s_bin, long long* s_rank) {
    const int t = threadIdx.x;
    unsigned int h[SEL_BPT];
    long long mine = 0;
#pragma unroll
    for (int q = 0; q < SEL_BPT; ++q) {
        h[q] = hist[SEL_BPT * t + q];
        mine += h[q];
    }
    long long incl = mine;  // inclusive scan over the wavefront, then wavefront totals through LDS
    for (int off = 1; off < FG_WAVE; off <<= 1) {
        const long long v = __shfl_up(incl, off, FG_WAVE);
        if (fg_lane() >= off) incl += v;
    }
    __syncthreads();
    if (fg_lane() == FG_WAVE - 1) red[fg_wave()] = incl;
    __syncthreads();
    long long before = incl - mine;
    for (int w = 0; w < fg_wave(); ++w) before += red[w];
    const long long rank = *s_rank;
    __syncthreads();
    if (rank >= before && rank < before + mine) {  // true for exactly one thread
        long long lo = before;
#pragma unroll
        for (int q = 0; q < SEL_BPT; ++q) {
            if (rank >= lo && rank < lo + h[q]) {
                *s_bin = SEL_BPT * t + q;
                *s_rank = rank - lo;
            }
            lo += h[q];
        }
    }
    __syncthreads();
}

// Calls f(key) for every live element, reading the norms 4 at a time (8 loads in flight per thread) when the
// arrays are suitably aligned; element order is irrelevant to the callers (they only count).
template <typename F>
__device__ __forceinline__ void for_each_live_key(const uint8_t* __restrict__ live, const float* __restrict__ gnorm, int n, F f) {
    const int t = threadIdx.x;
    const bool vec = (((uintptr_t)gnorm & 15) == 0) && (!live || ((uintptr_t)live & 3) == 0);
    int done = 0;
    if (vec) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const int n4 = n >> 2;
        for (int q0 = t; q0 < n4; q0 += 2 * SEL_THREADS) {
            const int q1 = q0 + SEL_THREADS;
            const bool has1 = q1 < n4;
            const f4 g0 = ((const f4*)gnorm)[q0];
            const f4 g1 = has1 ? ((const f4*)gnorm)[q1] : g0;
            const uint32_t l0 = live ? ((const uint32_t*)live)[q0] : 0x01010101u;
            const uint32_t l1 = live ? (has1 ? ((const uint32_t*)live)[q1] : 0u) : (has1 ? 0x01010101u : 0u);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((l0 >> (8 * e)) & 0xFFu) f(order_key(g0[e]));
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((l1 >> (8 * e)) & 0xFFu) f(order_key(g1[e]));
        }
        done = n4 << 2;
    }
    for (int j = done + t; j < n; j += SEL_THREADS)
        if (live ? live[j] != 0 : true) f(order_key(gnorm[j]));
}

__global__ __launch_bounds__(SEL_THREADS) void select_tau_kernel(const uint8_t* __restrict__ live,
                                                                 const float* __restrict__ gnorm, int n, float p_grad,
                                                                 UpdHeader* __restrict__ hdr, int64_t* __restrict__ stats) {
    __shared__ unsigned int hist[SEL_BINS];
    __shared__ uint32_t park[SEL_PARK];
    __shared__ long long red[16];
    __shared__ uint32_t s_bin;
    __shared__ long long s_rank;
    __shared__ unsigned int s_parked;
    const int t = threadIdx.x;
    // pass 0: top 11 bits of every live key; the histogram total is the live count m
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
    if (t == 0) s_parked = 0;
    __syncthreads();
    for_each_live_key(live, gnorm, n, [&](uint32_t kj) { atomicAdd(&hist[kj >> 21], 1u); });
    __syncthreads();
    long long c = 0;
#pragma unroll
    for (int q = 0; q < SEL_BPT; ++q) c += hist[SEL_BPT * t + q];
    const long long m = fg_block_sum(c, red);
    const long long k = (long long)floor((double)p_grad * (double)m);
    if (t == 0) {
        hdr->m_live = m;
        hdr->n_admit = 0;
        if (stats) stats[0] = stats[1] = stats[2] = stats[3] = 0;
    }
    if (k <= 0 || k >= m) {
        if (t == 0) {
            hdr->mode = k <= 0 ? 0 : 2;
            hdr->tau_key = 0;
        }
        return;
    }
    if (t == 0) s_rank = k;
    __syncthreads();
    select_bin(hist, red, &s_bin, &s_rank);
    const uint32_t d0 = s_bin;
    // pass 1: middle 11 bits of the keys whose top digit is d0; park those keys in LDS
    __syncthreads();
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
    __syncthreads();
    for_each_live_key(live, gnorm, n, [&](uint32_t kj) {
        if ((kj >> 21) != d0) return;
        atomicAdd(&hist[(kj >> 10) & 2047u], 1u);
        const unsigned int at = atomicAdd(&s_parked, 1u);
        if (at < SEL_PARK) park[at] = kj;
    });
    __syncthreads();
    select_bin(hist, red, &s_bin, &s_rank);
    const uint32_t d1 = s_bin;
    const uint32_t hi = (d0 << 21) | (d1 << 10);
    const unsigned int parked = s_parked;
    // pass 2: low 10 bits of the keys whose upper 22 bits are (d0, d1)
    __syncthreads();
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
    __syncthreads();
    if (parked <= SEL_PARK) {
        for (unsigned int i = t; i < parked; i += SEL_THREADS)
            if ((park[i] & 0xFFFFFC00u) == hi) atomicAdd(&hist[park[i] & 1023u], 1u);
    } else {
        for_each_live_key(live, gnorm, n, [&](uint32_t kj) {
            if ((kj & 0xFFFFFC00u) == hi) atomicAdd(&hist[kj & 1023u], 1u);
        });
    }
    __syncthreads();
    select_bin(hist, red, &s_bin, &s_rank);
    if (t == 0) {
        hdr->mode = 1;
        hdr->tau_key = hi | s_bin;
    }
}

// The same selection for up to 4096 * V elements with every key held in registers: one round of loads, all in
// flight at once, then the three digit passes run from registers. V = 4-key vectors per thread. Needs n >= 4,
// gnorm aligned to 16 bytes and live (if given) to 4.
template <int V>
__global__ __launch_bounds__(SEL_THREADS) void select_tau_reg_kernel(const uint8_t* __restrict__ live,
                                                                     const float* __restrict__ gnorm, int n, float p_grad,
                                                                     UpdHeader* __restrict__ hdr, int64_t* __restrict__ stats) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ unsigned int hist[SEL_BINS];
    __shared__ long long red[16];
    __shared__ uint32_t s_bin;
    __shared__ long long s_rank;
    const int t = threadIdx.x;
    const int nfull = n >> 2;
    f4 g[V];
    uint32_t lv[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {  // a vector past the end re-reads vector 0 and is masked below
        const int q = t + v * SEL_THREADS;
        const int qc = q < nfull ? q : 0;
        g[v] = ((const f4*)gnorm)[qc];
        lv[v] = live ? ((const uint32_t*)live)[qc] : 0x01010101u;
    }
    const int jt = (nfull << 2) + t;  // the up to three elements after the last whole vector
    const bool has_tail = t < 3 && jt < n;
    const uint32_t tail_key = has_tail ? order_key(gnorm[jt]) : 0u;
    const bool tail_live = has_tail && (live ? live[jt] != 0 : true);
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
    uint32_t key[V][4];
    uint64_t alive = 0;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const bool in = t + v * SEL_THREADS < nfull;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            key[v][e] = order_key(g[v][e]);
            if (in && ((lv[v] >> (8 * e)) & 0xFFu)) alive |= 1ull << (4 * v + e);
        }
    }
    __syncthreads();
    // pass 0: top 11 bits; the histogram total is the live count m
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if ((alive >> (4 * v + e)) & 1ull) atomicAdd(&hist[key[v][e] >> 21], 1u);
    if (tail_live) atomicAdd(&hist[tail_key >> 21], 1u);
    __syncthreads();
    long long c = 0;
#pragma unroll
    for (int q = 0; q < SEL_BPT; ++q) c += hist[SEL_BPT * t + q];
    const long long m = fg_block_sum(c, red);
    const long long k = (long long)floor((double)p_grad * (double)m);
    if (t == 0) {
        hdr->m_live = m;
        hdr->n_admit = 0;
        if (stats) stats[0] = stats[1] = stats[2] = stats[3] = 0;
    }
    if (k <= 0 || k >= m) {
        if (t == 0) {
            hdr->mode = k <= 0 ? 0 : 2;
            hdr->tau_key = 0;
        }
        return;
    }
    if (t == 0) s_rank = k;
    __syncthreads();
    select_bin(hist, red, &s_bin, &s_rank);
    const uint32_t d0 = s_bin;
    // pass 1: middle 11 bits of the keys whose top digit is d0
    __syncthreads();
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
    __syncthreads();
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (((alive >> (4 * v + e)) & 1ull) && (key[v][e] >> 21) == d0) atomicAdd(&hist[(key[v][e] >> 10) & 2047u], 1u);
    if (tail_live && (tail_key >> 21) == d0) atomicAdd(&hist[(tail_key >> 10) & 2047u], 1u);
    __syncthreads();
    select_bin(hist, red, &s_bin, &s_rank);
    const uint32_t hi = (d0 << 21) | (s_bin << 10);
    // pass 2: low 10 bits of the keys whose upper 22 bits are fixed by now
    __syncthreads();
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
    __syncthreads();
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (((alive >> (4 * v + e)) & 1ull) && (key[v][e] & 0xFFFFFC00u) == hi) atomicAdd(&hist[key[v][e] & 1023u], 1u);
    if (tail_live && (tail_key & 0xFFFFFC00u) == hi) atomicAdd(&hist[tail_key & 1023u], 1u);
    __syncthreads();
    select_bin(hist, red, &s_bin, &s_rank);
    if (t == 0) {
        hdr->mode = 1;
        hdr->tau_key = hi | s_bin;
    }
}

struct CacheRW {
    int32_t* map;
    int32_t* slot_node;
    int32_t* slot_stamp;
    const int64_t* head;  // current ring header
    int64_t* head_next;   // where an update leaves the advanced header (the two swap roles after every update)
    int64_t capacity;
    int64_t num_nodes;
    int64_t iter;
    int32_t t_stale;
};

__global__ __launch_bounds__(FG_SCAN_BLOCK) void classify_update_kernel(
    CacheRW c, const int32_t* __restrict__ ids, int n, const uint8_t* __restrict__ live,
    const uint8_t* __restrict__ hit, const float* __restrict__ gnorm, const UpdHeader* __restrict__ hdr,
    uint8_t* __restrict__ admit_flag, int32_t* __restrict__ blk_counts, int64_t* __restrict__ stats) {
    const int j = blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    bool admit = false, evict = false;
    if (j < n && (live ? live[j] != 0 : true)) {
        const int mode = hdr->mode;
        const bool low = mode == 2 || (mode == 1 && order_key(gnorm[j]) < hdr->tau_key);
        const bool is_hit = hit[j] != 0;
        const int32_t v = ids[j];
        const bool v_ok = v >= 0 && v < c.num_nodes;
        if (is_hit && !low && v_ok) {
            c.map[v] = -1;
            evict = true;
        }
        admit = !is_hit && low && v_ok;
    }
    if (j < n) admit_flag[j] = admit ? 1 : 0;
    const int n_admit = __syncthreads_count(admit);
    const int n_evict = __syncthreads_count(evict);
    if (threadIdx.x == 0) {
        blk_counts[blockIdx.x] = n_admit;
        if (stats && n_evict) atomicAdd((unsigned long long*)&stats[1], (unsigned long long)n_evict);
    }
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void assign_slots_kernel(
    CacheRW c, const int32_t* __restrict__ ids, int n, const uint8_t* __restrict__ admit_flag,
    const int32_t* __restrict__ blk_counts, UpdHeader* __restrict__ hdr, int32_t* __restrict__ admit_pos,
    int32_t* __restrict__ admit_slot, int64_t* __restrict__ stats) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    long long before = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += FG_SCAN_BLOCK) before += blk_counts[b];
    before = fg_block_sum(before, red);
    const int j = blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    const bool admit = j < n && admit_flag[j] != 0;
    int total;
    const long long rank = before + fg_block_rank(admit, total, sc);
    bool overwrote = false;
    if (admit && rank < c.capacity) {
        const int64_t head = *c.head;
        const int32_t s = (int32_t)((head + rank) % c.capacity);
        const int32_t v = ids[j];
        const int32_t old = c.slot_node[s];
        if (old >= 0 && old < c.num_nodes && c.map[old] == s) {
            const int64_t age = c.iter + 1 - (int64_t)c.slot_stamp[s];
            overwrote = age >= 1 && age <= (int64_t)c.t_stale;
        }
        c.slot_node[s] = v;
        c.slot_stamp[s] = (int32_t)c.iter;
        c.map[v] = s;
        admit_pos[rank] = j;
        admit_slot[rank] = s;
    }
    const int n_over = __syncthreads_count(overwrote);
    if (threadIdx.x == 0) {
        if (stats && n_over) atomicAdd((unsigned long long*)&stats[2], (unsigned long long)n_over);
        if (blockIdx.x == gridDim.x - 1) {
            const long long all = before + total;
            const long long in = all < c.capacity ? all : c.capacity;
            hdr->n_admit = in;
            *c.head_next = (*c.head + in) % c.capacity;
            if (stats) {
                stats[0] = in;
                stats[3] = all - in;
            }
        }
    }
}

struct UpdWs {
    size_t hdr, flag, blk, pos, slot, total;
};
UpdWs upd_layout(int64_t n) {
    UpdWs w;
    const int64_t nb = fg_ceil_div(n > 0 ? n : 1, FG_SCAN_BLOCK);
    w.hdr = 0;
    w.flag = 256;
    w.blk = w.flag + fg_align_up((size_t)n, 256);
    w.pos = w.blk + fg_align_up((size_t)nb * 4, 256);
    w.slot = w.pos + fg_align_up((size_t)n * 4, 256);
    w.total = w.slot + fg_align_up((size_t)n * 4, 256);
    return w;
}

// ---- export -----------------------------------------------------------------------------------------------

__global__ __launch_bounds__(FG_SCAN_BLOCK) void export_flag_kernel(CacheRW c, uint8_t* __restrict__ flag,
                                                                    int32_t* __restrict__ blk_counts) {
    const int64_t s = (int64_t)blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    bool valid = false;
    if (s < c.capacity) {
        const int32_t v = c.slot_node[s];
        if (v >= 0 && v < c.num_nodes && c.map[v] == (int32_t)s) {
            const int64_t age = c.iter - (int64_t)c.slot_stamp[s];
            valid = age >= 1 && age <= (int64_t)c.t_stale;
        }
        flag[s] = valid ? 1 : 0;
    }
    const int cnt = __syncthreads_count(valid);
    if (threadIdx.x == 0) blk_counts[blockIdx.x] = cnt;
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void export_write_kernel(CacheRW c, const uint8_t* __restrict__ flag,
                                                                     const int32_t* __restrict__ blk_counts,
                                                                     int32_t* __restrict__ nodes,
                                                                     int32_t* __restrict__ slots,
                                                                     int32_t* __restrict__ stamps,
                                                                     int64_t* __restrict__ count_out,
                                                                     int64_t* __restrict__ head_out) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    long long before = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += FG_SCAN_BLOCK) before += blk_counts[b];
    before = fg_block_sum(before, red);
    const int64_t s = (int64_t)blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    const bool valid = s < c.capacity && flag[s] != 0;
    int total;
    const long long rank = before + fg_block_rank(valid, total, sc);
    if (valid) {
        if (nodes) nodes[rank] = c.slot_node[s];
        if (slots) slots[rank] = (int32_t)s;
        if (stamps) stamps[rank] = c.slot_stamp[s];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        *count_out = before + total;
        if (head_out) *head_out = *c.head;
    }
}

fg_status_t layer_of(const fg_cache_t* cache, int32_t layer, const char* who, const fg_layer** out) {
    if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "%s: cache is NULL", who);
    if (layer < 1 || layer > cache->n_layers)
        FG_FAIL(FG_ERR_SHAPE, "%s: layer %d outside the cached layers 1..%d", who, layer, cache->n_layers);
    *out = &cache->layers[layer - 1];
    return FG_OK;
}

void free_layers(fg_cache_t* c) {
    if (!c) return;
    if (c->layers) {
        for (int i = 0; i < c->n_layers; ++i) {
            fg_layer& l = c->layers[i];
            if (l.map) (void)hipFree(l.map);
            if (l.slot_node) (void)hipFree(l.slot_node);
            if (l.slot_stamp) (void)hipFree(l.slot_stamp);
            if (l.table) (void)hipFree(l.table);
            if (l.head) (void)hipFree(l.head);
        }
        delete[] c->layers;
    }
    delete c;
}

}  // namespace

size_t fg_ws_cache_update_bytes(int64_t n) { return upd_layout(n).total; }
size_t fg_ws_export_bytes(int64_t capacity) {
    return fg_align_up((size_t)capacity, 256) + fg_align_up((size_t)fg_ceil_div(capacity > 0 ? capacity : 1, FG_SCAN_BLOCK) * 4, 256);
}

extern "C" fg_status_t fg_cache_clear(fg_cache_t* cache, void* stream) {
    if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_clear: cache is NULL");
    hipStream_t st = (hipStream_t)stream;
    for (int i = 0; i < cache->n_layers; ++i) {
        fg_layer& l = cache->layers[i];
        fg_status_t rc;
        if ((rc = fg_launch_fill_i32(l.map, cache->num_nodes, -1, st)) != FG_OK) return rc;
        if ((rc = fg_launch_fill_i32(l.slot_node, l.capacity, -1, st)) != FG_OK) return rc;
        if ((rc = fg_launch_fill_i32(l.slot_stamp, l.capacity, 0, st)) != FG_OK) return rc;
        if ((rc = fg_launch_fill_i32((int32_t*)l.head, 4, 0, st)) != FG_OK) return rc;
        l.head_cur = 0;
        l.last_iter = INT64_MIN;
    }
    fg_clear_error();
    return FG_OK;
}

extern "C" fg_status_t fg_cache_create(fg_cache_t** out, int64_t num_nodes, int32_t n_layers, const int64_t* capacity,
                                       const int32_t* dim, fg_dtype_t dtype, int32_t t_stale, void* stream) {
    if (!out) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_create: out is NULL");
    *out = nullptr;
    if (num_nodes <= 0 || num_nodes > INT32_MAX)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_create: num_nodes = %lld must be in 1..2^31-1", (long long)num_nodes);
    if (n_layers < 0 || (n_layers > 0 && (!capacity || !dim)))
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_create: n_layers = %d needs capacity and dim arrays", n_layers);
    if (t_stale < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_create: t_stale = %d is negative", t_stale);
    const int esz = fg_dtype_size(dtype);
    if (!esz) FG_FAIL(FG_ERR_DTYPE, "fg_cache_create: unknown element type %d", (int)dtype);
    for (int i = 0; i < n_layers; ++i) {
        if (capacity[i] <= 0 || capacity[i] > INT32_MAX)
            FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_create: capacity[%d] = %lld must be in 1..2^31-1", i, (long long)capacity[i]);
        if (dim[i] <= 0 || ((int64_t)dim[i] * esz) % 16)
            FG_FAIL(FG_ERR_SHAPE, "fg_cache_create: dim[%d] = %d must give rows that are a multiple of 16 bytes", i, dim[i]);
    }
    fg_cache_t* c = new fg_cache_t();
    c->num_nodes = num_nodes;
    c->n_layers = n_layers;
    c->dtype = dtype;
    c->t_stale = t_stale;
    c->layers = n_layers ? new fg_layer[n_layers]() : nullptr;
    for (int i = 0; i < n_layers; ++i) {
        fg_layer& l = c->layers[i];
        l.capacity = capacity[i];
        l.dim = dim[i];
        hipError_t e = hipMalloc((void**)&l.map, (size_t)num_nodes * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&l.slot_node, (size_t)l.capacity * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&l.slot_stamp, (size_t)l.capacity * 4);
        if (e == hipSuccess) e = hipMalloc(&l.table, (size_t)l.capacity * l.dim * esz);
        if (e == hipSuccess) e = hipMalloc((void**)&l.head, 16);
        if (e != hipSuccess) {
            free_layers(c);
            (void)hipGetLastError();
            FG_FAIL(e == hipErrorOutOfMemory ? FG_ERR_OOM : FG_ERR_HIP, "fg_cache_create: allocation for layer %d failed: %s",
                    i + 1, hipGetErrorString(e));
        }
    }
    fg_status_t rc = fg_cache_clear(c, stream);
    if (rc != FG_OK) {
        free_layers(c);
        return rc;
    }
    *out = c;
    return FG_OK;
}

extern "C" fg_status_t fg_cache_destroy(fg_cache_t* cache) {
    if (!cache) return FG_OK;
    (void)hipDeviceSynchronize();
    free_layers(cache);
    return FG_OK;
}

extern "C" const void* fg_cache_table(const fg_cache_t* cache, int32_t layer) {
    const fg_layer* l;
    if (layer_of(cache, layer, "fg_cache_table", &l) != FG_OK) return nullptr;
    return l->table;
}

extern "C" fg_status_t fg_cache_set_t_stale(fg_cache_t* cache, int32_t t_stale) {
    if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_set_t_stale: cache is NULL");
    if (t_stale < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_set_t_stale: t_stale = %d is negative", t_stale);
    cache->t_stale = t_stale;
    return FG_OK;
}

extern "C" fg_status_t fg_cache_export(const fg_cache_t* cache, int32_t layer, int64_t iter, int32_t* nodes_dev,
                                       int32_t* slots_dev, int32_t* stamps_dev, int64_t* count_dev, int64_t* head_dev,
                                       void* ws_dev, size_t ws_bytes, void* stream) {
    const fg_layer* l;
    fg_status_t rc = layer_of(cache, layer, "fg_cache_export", &l);
    if (rc != FG_OK) return rc;
    if (!count_dev) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_export: count_dev is NULL");
    const size_t need = fg_ws_export_bytes(l->capacity);
    if (!ws_dev || ws_bytes < need) FG_FAIL(FG_ERR_SHAPE, "fg_cache_export: workspace of %zu bytes given, %zu needed", ws_bytes, need);
    fg_clear_error();
    CacheRW c{l->map, l->slot_node, l->slot_stamp, l->head + l->head_cur, nullptr, l->capacity, cache->num_nodes, iter, cache->t_stale};
    uint8_t* flag = (uint8_t*)ws_dev;
    int32_t* blk = (int32_t*)((char*)ws_dev + fg_align_up((size_t)l->capacity, 256));
    const int nb = (int)fg_ceil_div(l->capacity, FG_SCAN_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(export_flag_kernel, dim3(nb), dim3(FG_SCAN_BLOCK), 0, st, c, flag, blk);
    FG_LAUNCH_CHECK("export_flag_kernel");
    hipLaunchKernelGGL(export_write_kernel, dim3(nb), dim3(FG_SCAN_BLOCK), 0, st, c, flag, blk, nodes_dev, slots_dev,
                       stamps_dev, count_dev, head_dev);
    FG_LAUNCH_CHECK("export_write_kernel");
    return FG_OK;
}

extern "C" fg_status_t fg_cache_update(fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev,
                                       int32_t n, const uint8_t* live_dev, const uint8_t* hit_dev,
                                       const float* gnorm_dev, float p_grad, const void* h_dev, int64_t h_stride,
                                       int64_t* stats_dev, void* ws_dev, size_t ws_bytes, void* stream) {
    const fg_layer* lc;
    fg_status_t rc = layer_of(cache, layer, "fg_cache_update", &lc);
    if (rc != FG_OK) return rc;
    fg_layer* l = &cache->layers[layer - 1];
    if (n < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_update: n = %d is negative", n);
    if (!(p_grad >= 0.0f && p_grad <= 1.0f)) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_update: p_grad = %g outside [0, 1]", (double)p_grad);
    if (n > 0 && (!ids_dev || !hit_dev || !gnorm_dev || !h_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_update: NULL pointer");
    const int64_t row_bytes = (int64_t)l->dim * fg_dtype_size(cache->dtype);
    if (h_stride < row_bytes) FG_FAIL(FG_ERR_SHAPE, "fg_cache_update: h_stride = %lld smaller than a cache row of %lld bytes", (long long)h_stride, (long long)row_bytes);
    if (((uintptr_t)h_dev | (uintptr_t)h_stride) & 15) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_update: h_dev and h_stride must be 16-byte aligned");
    if (iter < l->last_iter) FG_FAIL(FG_ERR_STATE, "fg_cache_update: iteration %lld after %lld: the counter must not go backwards", (long long)iter, (long long)l->last_iter);
    if (iter < 0 || iter > INT32_MAX - 1) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_update: iteration %lld out of range", (long long)iter);
    const UpdWs w = upd_layout(n);
    if (!ws_dev || ws_bytes < w.total) FG_FAIL(FG_ERR_SHAPE, "fg_cache_update: workspace of %zu bytes given, %zu needed", ws_bytes, w.total);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_update: workspace must be 16-byte aligned");
    fg_clear_error();
    l->last_iter = iter;
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)ws_dev;
    UpdHeader* hdr = (UpdHeader*)(ws + w.hdr);
    uint8_t* flag = (uint8_t*)(ws + w.flag);
    int32_t* blk = (int32_t*)(ws + w.blk);
    int32_t* apos = (int32_t*)(ws + w.pos);
    int32_t* aslot = (int32_t*)(ws + w.slot);
    CacheRW c{l->map, l->slot_node, l->slot_stamp, l->head + l->head_cur, l->head + (l->head_cur ^ 1), l->capacity, cache->num_nodes, iter, cache->t_stale};
    const bool aligned = (((uintptr_t)gnorm_dev & 15) == 0) && (((uintptr_t)live_dev & 3) == 0);
#define FG_SEL_REG(V) hipLaunchKernelGGL(select_tau_reg_kernel<V>, dim3(1), dim3(SEL_THREADS), 0, st, live_dev, gnorm_dev, n, p_grad, hdr, stats_dev)
    if (!aligned || n < 4 || n > 16 * 4 * SEL_THREADS)
        hipLaunchKernelGGL(select_tau_kernel, dim3(1), dim3(SEL_THREADS), 0, st, live_dev, gnorm_dev, n, p_grad, hdr, stats_dev);
    else if (n <= 1 * 4 * SEL_THREADS) FG_SEL_REG(1);
    else if (n <= 2 * 4 * SEL_THREADS) FG_SEL_REG(2);
    else if (n <= 4 * 4 * SEL_THREADS) FG_SEL_REG(4);
    else if (n <= 8 * 4 * SEL_THREADS) FG_SEL_REG(8);
    else FG_SEL_REG(16);
#undef FG_SEL_REG
    FG_LAUNCH_CHECK("select_tau_kernel");
    if (n == 0) return FG_OK;
    const int nb = (int)fg_ceil_div(n, FG_SCAN_BLOCK);
    hipLaunchKernelGGL(classify_update_kernel, dim3(nb), dim3(FG_SCAN_BLOCK), 0, st, c, ids_dev, n, live_dev, hit_dev,
                       gnorm_dev, hdr, flag, blk, stats_dev);
    FG_LAUNCH_CHECK("classify_update_kernel");
    hipLaunchKernelGGL(assign_slots_kernel, dim3(nb), dim3(FG_SCAN_BLOCK), 0, st, c, ids_dev, n, flag, blk, hdr, apos,
                       aslot, stats_dev);
    FG_LAUNCH_CHECK("assign_slots_kernel");
    rc = fg_launch_gather(h_dev, n, h_stride, row_bytes, apos, aslot, &hdr->n_admit, n < l->capacity ? n : l->capacity,
                          l->table, l->capacity, row_bytes, FG_TABLE_HBM_REUSED, st);
    if (rc != FG_OK) return rc;
    l->head_cur ^= 1;  // the advanced header written by assign_slots is the current one from here on
    return FG_OK;
}
