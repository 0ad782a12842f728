// The historical embedding cache (Section 4.2, embedding side) and its Update (Algorithm 1, last loop;
// admission and check-out by gradient norm, Section 4.1.1; staleness bound, Section 4.1.2).
//
// State per cached layer, all in HBM: map[num_nodes] (slot of a node or -1), table[capacity x dim],
// slot_node[capacity], slot_stamp[capacity], head, and 16 KB of selection scratch. The tables of all layers
// lie in one buffer, from its left end in layer order; raw features can be placed from its right end (the
// bidirectional cache of Section 4.2, see the feature side at the end of this file). A node v is usable at
// iteration i iff
//   s = map[v] >= 0, slot_node[s] == v and 1 <= i - slot_stamp[s] <= t_stale.
// The back-pointer test makes every location single-writer during an update: admitting into a slot never
// touches the previous owner's map entry, a check-out only writes the node's own map entry, and the slots
// handed out in one update are distinct. The result is therefore the same as the sequential procedure.
//
// Update = 5 launches for any number of layers (a workgroup finds its layer from its index), no host
// synchronisation and no waiting between workgroups:
//   1. digit 0       histogram of the top 11 bits of the order-preserving integer image of the live nodes' norms
//   2. digit 1       every workgroup derives m, k = floor(p_grad*m) and the first digit of the norm of rank k from
//                    the finished histogram, then histograms the next 11 bits of its keys that carry that digit
//                    and appends those keys to the layer's survivor list
//   3. classify      every workgroup finishes the selection (second digit from the histogram, last 10 bits from
//                    the survivor list): tau, exactly. Then: check out hits that are not below tau; flag
//                    admissible normal nodes; count per workgroup
//   4. assign_slots  rank admissible nodes in position order (ballot ranks + preceding workgroups' counts),
//                    hand out ring slots head + rank, write slot_node / slot_stamp / map, list (position, slot);
//                    the last workgroup leaves the advanced header in the spare header cell
//   5. row copy      table[slot] = h[position]
// With the access-aware policy (a layer given estimates of saved accesses and a budget smaller than what is admissible;
// Section 7.4 names the policy, the rule is this build's reading) launch 3 also histograms the estimates of the
// admissible nodes and one more launch between 3 and 4 (rank_saving) finds the estimate of rank `room` from the top,
// re-flags every admissible node as in / tie / out and counts per workgroup; launch 4 then lets the first ties in
// position order fill what the larger estimates leave of the room.
#include "common.h"
#include "scan.h"

namespace {

struct UpdHeader {        // lives at the start of a layer's update workspace
    uint32_t tau_key;     // order-preserving key of tau
    int32_t mode;         // 0: nothing is below tau, 1: compare with tau_key, 2: everything is below tau
    int64_t n_admit;      // rows to copy (<= capacity)
    int64_t m_live;
    int64_t n_cand;       // access-aware policy: admissible nodes, and how many of those whose estimate equals the
    int64_t tie_room;     //   threshold estimate still fit (-1: every admissible node fits)
};

__device__ __forceinline__ int clamp_saving(int32_t a) { return a < 0 ? 0 : (a > 2047 ? 2047 : a); }

__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int SEL_THREADS = 1024;
constexpr int SEL_BINS = 2048;
constexpr int SEL_BPT = SEL_BINS / SEL_THREADS;  // bins owned by a thread in the scan
constexpr int SEL_CHUNK = 4 * SEL_THREADS;       // keys per workgroup in the histogram launches
constexpr int FG_MAX_UPD_LAYERS = 8;

// Selection scratch of a layer, owned by the cache. All-zero between updates: launch 4 clears it again.
struct SelState {
    unsigned int hist0[SEL_BINS];
    unsigned int hist1[SEL_BINS];
    unsigned int n_surv;
    unsigned int pad[3];
    unsigned int hist2[SEL_BINS];  // estimates of saved accesses of the admissible nodes (access-aware policy)
};

static_assert(SEL_BINS == 2048, "clamp_saving saturates the estimates at the last bin");

struct CacheRW {
    int32_t* map;
    int32_t* slot_node;
    int32_t* slot_stamp;
    const int64_t* head;  // current ring header
    int64_t* head_next;   // where an update leaves the advanced header (the two swap roles after every update)
    int64_t* used;        // slots written at least once (what the ring has overwritten of the shared buffer)
    int64_t capacity;
    int64_t num_nodes;
    int64_t iter;
    int32_t t_stale;
};

struct UpdLayer {
    CacheRW c;
    const int32_t* ids;
    const uint8_t* live;
    const uint8_t* hit;
    const float* gnorm;
    int64_t* stats;
    SelState* sel;
    UpdHeader* hdr;
    uint8_t* flag;       // per position: 0 not admitted, 1 admissible (in position order while there is room), 2 in for sure
    int32_t* blk;        // flag-1 nodes per workgroup of launch 3
    int32_t* blk_sure;   // flag-2 nodes per workgroup (access-aware policy)
    const int32_t* saving;  // estimates of saved accesses by position, or NULL
    int64_t room;        // rows this update may admit (<= capacity)
    int32_t* apos;       // admitted positions; before launch 4 the same memory holds the survivor keys
    int32_t* aslot;      // their slots
    const char* h;
    int64_t h_stride;
    char* table;
    int64_t row_bytes;
    int32_t n;           // positions of the layer: the caller's bound ...
    const int64_t* n_dev;  // ... and, if non-null, the count in device memory (positions at or beyond it are not live)
    float p_grad;
};

// positions of the layer that exist: the device-side count where the caller gave one, never above the bound
__device__ __forceinline__ int upd_count(const UpdLayer& L) {
    if (!L.n_dev) return L.n;
    const int64_t c = *L.n_dev;
    return c < 0 ? 0 : (c < (int64_t)L.n ? (int)c : L.n);
}

struct UpdBatch {
    int32_t n_layers;
    int32_t sel_first[FG_MAX_UPD_LAYERS + 1];   // first workgroup of each layer in launches 1 and 2
    int32_t scan_first[FG_MAX_UPD_LAYERS + 1];  // the same for launches 3 and 4
    UpdLayer l[FG_MAX_UPD_LAYERS];
};

__device__ __forceinline__ int layer_of_block(const int32_t* first, int n_layers, int b, int& local) {
    int l = 0;
    while (l + 1 < n_layers && b >= first[l + 1]) ++l;
    local = b - first[l];
    return l;
}

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

// Calls f(key) for every live element of chunk `chunk` (SEL_CHUNK elements), reading the norms 4 at a time when
// the arrays are suitably aligned; element order is irrelevant to the callers (they only count).
template <typename F>
__device__ __forceinline__ void for_each_live_key(const uint8_t* __restrict__ live, const float* __restrict__ gnorm, int n,
                                                  int chunk, F f) {
    const int t = threadIdx.x;
    const int begin = chunk * SEL_CHUNK;
    const int len = n - begin < SEL_CHUNK ? n - begin : SEL_CHUNK;
    if (len <= 0) return;
    gnorm += begin;
    if (live) live += begin;
    const bool vec = (((uintptr_t)gnorm & 15) == 0) && (!live || ((uintptr_t)live & 3) == 0);
    int done = 0;
    if (vec) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const int n4 = len >> 2;
        if (t < n4) {  // SEL_CHUNK = 4 * SEL_THREADS: one vector per thread
            const f4 g = ((const f4*)gnorm)[t];
            const uint32_t l4 = live ? ((const uint32_t*)live)[t] : 0x01010101u;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((l4 >> (8 * e)) & 0xFFu) f(order_key(g[e]));
        }
        done = n4 << 2;
    }
    for (int j = done + t; j < len; j += SEL_THREADS)
        if (live ? live[j] != 0 : true) f(order_key(gnorm[j]));
}

// From the finished first histogram: m (live count), k = floor(p_grad * m) and, unless k is degenerate, the first
// digit d0 of the key of rank k; *s_rank is left holding the rank among the keys with that digit. Returns the
// mode (0: nothing is below tau, 2: everything is, 1: tau has to be found). Every thread gets the same values.
__device__ __forceinline__ int first_digit(const SelState* __restrict__ S, float p_grad, unsigned int* hist, long long* red,
                                           uint32_t* s_bin, long long* s_rank, uint32_t& d0, long long& m) {
    const int t = threadIdx.x;
    __syncthreads();
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = S->hist0[b];
    __syncthreads();
    long long c = 0;
#pragma unroll
    for (int q = 0; q < SEL_BPT; ++q) c += hist[SEL_BPT * t + q];
    m = fg_block_sum(c, red);
    const long long k = (long long)floor((double)p_grad * (double)m);
    d0 = 0;
    if (k <= 0) return 0;
    if (k >= m) return 2;
    if (t == 0) *s_rank = k;
    __syncthreads();
    select_bin(hist, red, s_bin, s_rank);
    d0 = *s_bin;
    return 1;
}

__global__ __launch_bounds__(SEL_THREADS) void update_digit0_kernel(UpdBatch B) {
    __shared__ unsigned int hist[SEL_BINS];
    int chunk;
    const UpdLayer& L = B.l[layer_of_block(B.sel_first, B.n_layers, blockIdx.x, chunk)];
    const int t = threadIdx.x;
    if (chunk == 0 && t == 0 && L.stats) L.stats[0] = L.stats[1] = L.stats[2] = L.stats[3] = 0;
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
    __syncthreads();
    for_each_live_key(L.live, L.gnorm, upd_count(L), chunk, [&](uint32_t kj) { atomicAdd(&hist[kj >> 21], 1u); });
    __syncthreads();
    for (int b = t; b < SEL_BINS; b += SEL_THREADS)
        if (hist[b]) atomicAdd(&L.sel->hist0[b], hist[b]);
}

__global__ __launch_bounds__(SEL_THREADS) void update_digit1_kernel(UpdBatch B) {
    __shared__ unsigned int hist[SEL_BINS];
    __shared__ uint32_t park[SEL_CHUNK];
    __shared__ long long red[16];
    __shared__ uint32_t s_bin;
    __shared__ long long s_rank;
    __shared__ unsigned int s_parked, s_base;
    int chunk;
    const UpdLayer& L = B.l[layer_of_block(B.sel_first, B.n_layers, blockIdx.x, chunk)];
    const int t = threadIdx.x;
    uint32_t d0;
    long long m;
    if (first_digit(L.sel, L.p_grad, hist, red, &s_bin, &s_rank, d0, m) != 1) return;  // uniform over the layer
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
    if (t == 0) s_parked = 0;
    __syncthreads();
    for_each_live_key(L.live, L.gnorm, upd_count(L), chunk, [&](uint32_t kj) {
        if ((kj >> 21) != d0) return;
        atomicAdd(&hist[(kj >> 10) & 2047u], 1u);
        park[atomicAdd(&s_parked, 1u)] = kj;  // a workgroup sees at most SEL_CHUNK keys
    });
    __syncthreads();
    const unsigned int parked = s_parked;
    if (t == 0 && parked) s_base = atomicAdd(&L.sel->n_surv, parked);
    for (int b = t; b < SEL_BINS; b += SEL_THREADS)
        if (hist[b]) atomicAdd(&L.sel->hist1[b], hist[b]);
    __syncthreads();
    uint32_t* survivors = (uint32_t*)L.apos;  // at most n keys in all
    for (unsigned int i = t; i < parked; i += SEL_THREADS) survivors[s_base + i] = park[i];
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void classify_update_kernel(UpdBatch B) {
    static_assert(FG_SCAN_BLOCK == SEL_THREADS, "the selection helpers assume this workgroup size");
    __shared__ unsigned int hist[SEL_BINS];
    __shared__ long long red[16];
    __shared__ uint32_t s_bin;
    __shared__ long long s_rank;
    int local;
    const UpdLayer& L = B.l[layer_of_block(B.scan_first, B.n_layers, blockIdx.x, local)];
    const CacheRW& c = L.c;
    const int t = threadIdx.x;
    // this thread's element first: the loads are in flight while the selection below runs
    const int j = local * FG_SCAN_BLOCK + t;
    const bool in = j < upd_count(L);
    const int jc = in ? j : 0;
    const uint8_t live_j = in ? (L.live ? L.live[jc] : (uint8_t)1) : (uint8_t)0;
    const uint32_t key_j = in ? order_key(L.gnorm[jc]) : 0u;
    const uint8_t hit_j = in ? L.hit[jc] : (uint8_t)0;
    const int32_t v = in ? L.ids[jc] : -1;
    // the rest of the selection, the same in every workgroup of the layer
    uint32_t d0, tau_key = 0;
    long long m;
    const int mode = first_digit(L.sel, L.p_grad, hist, red, &s_bin, &s_rank, d0, m);
    if (mode == 1) {
        __syncthreads();
        for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = L.sel->hist1[b];
        __syncthreads();
        select_bin(hist, red, &s_bin, &s_rank);
        const uint32_t hi = (d0 << 21) | (s_bin << 10);
        __syncthreads();
        for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
        __syncthreads();
        const unsigned int n_surv = L.sel->n_surv;
        const uint32_t* survivors = (const uint32_t*)L.apos;
        for (unsigned int i = t; i < n_surv; i += SEL_THREADS) {
            const uint32_t kj = survivors[i];
            if ((kj & 0xFFFFFC00u) == hi) atomicAdd(&hist[kj & 1023u], 1u);
        }
        __syncthreads();
        select_bin(hist, red, &s_bin, &s_rank);
        tau_key = hi | s_bin;
    }
    if (local == 0 && t == 0) {
        L.hdr->mode = mode;
        L.hdr->tau_key = tau_key;
        L.hdr->m_live = m;
    }
    bool admit = false, evict = false;
    if (live_j != 0) {
        const bool low = mode == 2 || (mode == 1 && key_j < tau_key);
        const bool is_hit = hit_j != 0;
        const bool v_ok = v >= 0 && v < c.num_nodes;
        if (is_hit && !low && v_ok) {
            c.map[v] = -1;
            evict = true;
        }
        admit = !is_hit && low && v_ok;
    }
    if (j < L.n) L.flag[j] = admit ? 1 : 0;
    const int n_admit = __syncthreads_count(admit);
    const int n_evict = __syncthreads_count(evict);
    if (t == 0) {
        L.blk[local] = n_admit;
        if (L.stats && n_evict) atomicAdd((unsigned long long*)&L.stats[1], (unsigned long long)n_evict);
    }
    if (L.saving) {  // uniform over the layer
        for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
        __syncthreads();
        if (admit) atomicAdd(&hist[clamp_saving(L.saving[j])], 1u);
        __syncthreads();
        for (int b = t; b < SEL_BINS; b += SEL_THREADS)
            if (hist[b]) atomicAdd(&L.sel->hist2[b], hist[b]);
    }
}

// Access-aware policy, between classify and assign_slots: with T admissible nodes and room for R < T of them, the R
// largest estimates get in, equal estimates in position order. Every workgroup finds the threshold estimate a* (rank
// T - R in ascending order) and how many nodes at a* still fit, then re-flags its nodes: above a* -> 2, at a* -> 1,
// below -> 0. With T <= R the flags stay as they are.
__global__ __launch_bounds__(FG_SCAN_BLOCK) void rank_saving_kernel(UpdBatch B) {
    __shared__ unsigned int hist[SEL_BINS];
    __shared__ long long red[16];
    __shared__ uint32_t s_bin;
    __shared__ long long s_rank;
    int local;
    const UpdLayer& L = B.l[layer_of_block(B.scan_first, B.n_layers, blockIdx.x, local)];
    if (!L.saving) return;
    const int t = threadIdx.x;
    const int j = local * FG_SCAN_BLOCK + t;
    const bool cand = j < L.n && L.flag[j] != 0;
    const int a_j = cand ? clamp_saving(L.saving[j]) : 0;
    for (int b = t; b < SEL_BINS; b += SEL_THREADS) hist[b] = L.sel->hist2[b];
    __syncthreads();
    long long c = 0;
#pragma unroll
    for (int q = 0; q < SEL_BPT; ++q) c += hist[SEL_BPT * t + q];
    const long long T = fg_block_sum(c, red);
    if (T <= L.room) {
        if (local == 0 && t == 0) {
            L.hdr->n_cand = T;
            L.hdr->tie_room = -1;
        }
        if (t == 0) L.blk_sure[local] = 0;
        return;
    }
    if (t == 0) s_rank = T - L.room;
    __syncthreads();
    select_bin(hist, red, &s_bin, &s_rank);
    const int a_star = (int)s_bin;
    const long long tie_room = (long long)hist[a_star] - s_rank;  // nodes at a* that get in
    const bool sure = cand && a_j > a_star, tie = cand && a_j == a_star;
    if (cand) L.flag[j] = sure ? 2 : (tie ? 1 : 0);
    const int n_sure = __syncthreads_count(sure);
    const int n_tie = __syncthreads_count(tie);
    if (t == 0) {
        L.blk_sure[local] = n_sure;
        L.blk[local] = n_tie;
        if (local == 0) {
            L.hdr->n_cand = T;
            L.hdr->tie_room = tie_room;
        }
    }
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void assign_slots_kernel(UpdBatch B) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    int local;
    const int layer = layer_of_block(B.scan_first, B.n_layers, blockIdx.x, local);
    const UpdLayer& L = B.l[layer];
    const CacheRW& c = L.c;
    const int n_local = B.scan_first[layer + 1] - B.scan_first[layer];
    if (local == 0)  // every workgroup of the layer has used the selection scratch in the previous launch
        for (int i = threadIdx.x; i < (int)(sizeof(SelState) / 4); i += FG_SCAN_BLOCK) ((unsigned int*)L.sel)[i] = 0;
    // this thread's element and the ring header first: in flight while the preceding workgroups' counts are added up
    const int j = local * FG_SCAN_BLOCK + threadIdx.x;
    const uint8_t flag_j = j < L.n ? L.flag[j] : (uint8_t)0;
    const int32_t v_j = j < L.n ? L.ids[j] : -1;
    const int64_t head = *c.head;
    long long before = 0;
    for (int b = threadIdx.x; b < local; b += FG_SCAN_BLOCK) before += L.blk[b];
    before = fg_block_sum(before, red);
    int total;
    long long rank = before + fg_block_rank(flag_j == 1, total, sc);  // among the flag-1 nodes, in position order
    long long room = L.room, n_cand = -1, sure_all = 0;
    bool admit = flag_j == 1 && rank < room;
    if (L.saving) {  // uniform over the layer: flag-2 nodes are in, flag-1 nodes share what is left of the room
        const long long tie_room = L.hdr->tie_room;
        n_cand = L.hdr->n_cand;
        if (tie_room >= 0) {
            long long sure_before = 0;
            for (int b = threadIdx.x; b < local; b += FG_SCAN_BLOCK) sure_before += L.blk_sure[b];
            sure_before = fg_block_sum(sure_before, red);
            int sure_total;
            const long long sure_rank = sure_before + fg_block_rank(flag_j == 2, sure_total, sc);
            const long long ties_in = rank < tie_room ? rank : tie_room;  // ties admitted before this position
            admit = flag_j == 2 || (flag_j == 1 && rank < tie_room);
            rank = sure_rank + ties_in;
            room = tie_room;
            sure_all = sure_before + sure_total;
        }
    }
    bool overwrote = false;
    if (admit) {
        const int32_t s = (int32_t)((head + rank) % c.capacity);
        const int32_t v = v_j;
        const int32_t old = c.slot_node[s];
        if (old >= 0 && old < c.num_nodes && c.map[old] == s) {
            const int64_t age = c.iter + 1 - (int64_t)c.slot_stamp[s];
            overwrote = age >= 1 && age <= (int64_t)c.t_stale;
        }
        c.slot_node[s] = v;
        c.slot_stamp[s] = (int32_t)c.iter;
        c.map[v] = s;
        L.apos[rank] = j;
        L.aslot[rank] = s;
    }
    const int n_over = __syncthreads_count(overwrote);
    if (threadIdx.x == 0) {
        if (L.stats && n_over) atomicAdd((unsigned long long*)&L.stats[2], (unsigned long long)n_over);
        if (local == n_local - 1) {
            const long long ties = before + total;
            const long long in = sure_all + (ties < room ? ties : room);
            const long long all = n_cand >= 0 ? n_cand : ties;
            L.hdr->n_admit = in;
            *c.head_next = (head + in) % c.capacity;
            const int64_t reach = head + in;  // the ring fills slots upwards until it first wraps
            if (reach >= c.capacity)
                *c.used = c.capacity;
            else if (reach > *c.used)
                *c.used = reach;
            if (L.stats) {
                L.stats[0] = in;
                L.stats[3] = all - in;
            }
        }
    }
}

struct UpdWs {
    size_t hdr, flag, blk, blk_sure, pos, slot, total;
};
UpdWs upd_layout(int64_t n) {
    UpdWs w;
    const int64_t nb = fg_ceil_div(n > 0 ? n : 1, FG_SCAN_BLOCK);
    w.hdr = 0;
    w.flag = 256;
    w.blk = w.flag + fg_align_up((size_t)n, 256);
    w.blk_sure = w.blk + fg_align_up((size_t)nb * 4, 256);
    w.pos = w.blk_sure + fg_align_up((size_t)nb * 4, 256);
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
            if (l.head) (void)hipFree(l.head);
            if (l.sel) (void)hipFree(l.sel);
        }
        delete[] c->layers;
    }
    if (c->buffer) (void)hipFree(c->buffer);
    if (c->feat_rank) (void)hipFree(c->feat_rank);
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
        if ((rc = fg_launch_fill_i32((int32_t*)l.head, 8, 0, st)) != FG_OK) return rc;
        if ((rc = fg_launch_fill_i32((int32_t*)l.sel, sizeof(SelState) / 4, 0, st)) != FG_OK) return rc;
        l.head_cur = 0;
        l.last_iter = INT64_MIN;
        l.copy_pending = false;
    }
    // an emptied ring has "written" nothing, so rows placed earlier would count as intact although embeddings
    // may have been written over them: the feature side is dropped with the embeddings
    if (cache->feat_rank && cache->n_feat > 0) {
        fg_status_t rc = fg_launch_fill_i32(cache->feat_rank, cache->num_nodes, -1, st);
        if (rc != FG_OK) return rc;
    }
    cache->n_feat = 0;
    cache->feat_row_bytes = 0;
    fg_clear_error();
    return FG_OK;
}

static fg_status_t create_cache(const char* who, fg_cache_t** out, int64_t num_nodes, int32_t n_layers, const int64_t* capacity,
                                const int32_t* dim, fg_dtype_t dtype, int32_t t_stale, int64_t buffer_bytes, void* stream);

extern "C" fg_status_t fg_cache_create(fg_cache_t** out, int64_t num_nodes, int32_t n_layers, const int64_t* capacity,
                                       const int32_t* dim, fg_dtype_t dtype, int32_t t_stale, void* stream) {
    return create_cache("fg_cache_create", out, num_nodes, n_layers, capacity, dim, dtype, t_stale, 0, stream);
}

extern "C" fg_status_t fg_cache_create_bidirectional(fg_cache_t** out, int64_t num_nodes, int32_t n_layers,
                                                     const int64_t* capacity, const int32_t* dim, fg_dtype_t dtype,
                                                     int32_t t_stale, int64_t buffer_bytes, void* stream) {
    if (out) *out = nullptr;
    if (buffer_bytes <= 0 || buffer_bytes % FG_RING_ALIGN)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_create_bidirectional: buffer_bytes = %lld must be a positive multiple of %lld",
                (long long)buffer_bytes, (long long)FG_RING_ALIGN);
    if (n_layers > FG_MAX_RINGS)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_create_bidirectional: at most %d cached layers share a buffer with features", FG_MAX_RINGS);
    return create_cache("fg_cache_create_bidirectional", out, num_nodes, n_layers, capacity, dim, dtype, t_stale, buffer_bytes, stream);
}

// buffer_bytes = 0: a buffer that just holds the rings
static fg_status_t create_cache(const char* who, fg_cache_t** out, int64_t num_nodes, int32_t n_layers, const int64_t* capacity,
                                const int32_t* dim, fg_dtype_t dtype, int32_t t_stale, int64_t buffer_bytes, void* stream) {
    if (!out) FG_FAIL(FG_ERR_INVALID_ARG, "%s: out is NULL", who);
    *out = nullptr;
    if (num_nodes <= 0 || num_nodes > INT32_MAX)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: num_nodes = %lld must be in 1..2^31-1", who, (long long)num_nodes);
    if (n_layers < 0 || (n_layers > 0 && (!capacity || !dim)))
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: n_layers = %d needs capacity and dim arrays", who, n_layers);
    if (t_stale < 0) FG_FAIL(FG_ERR_INVALID_ARG, "%s: t_stale = %d is negative", who, t_stale);
    const int esz = fg_dtype_size(dtype);
    if (!esz) FG_FAIL(FG_ERR_DTYPE, "%s: unknown element type %d", who, (int)dtype);
    int64_t rings_end = 0;  // rings from the left end of the buffer, in layer order, each start aligned
    for (int i = 0; i < n_layers; ++i) {
        if (capacity[i] <= 0 || capacity[i] > INT32_MAX)
            FG_FAIL(FG_ERR_INVALID_ARG, "%s: capacity[%d] = %lld must be in 1..2^31-1", who, i, (long long)capacity[i]);
        if (dim[i] <= 0 || ((int64_t)dim[i] * esz) % 16)
            FG_FAIL(FG_ERR_SHAPE, "%s: dim[%d] = %d must give rows that are a multiple of 16 bytes", who, i, dim[i]);
        rings_end = (int64_t)fg_align_up((size_t)rings_end, FG_RING_ALIGN) + capacity[i] * dim[i] * esz;
    }
    if (buffer_bytes == 0) buffer_bytes = (int64_t)fg_align_up((size_t)rings_end, FG_RING_ALIGN);
    if (buffer_bytes < rings_end)
        FG_FAIL(FG_ERR_SHAPE, "%s: buffer_bytes = %lld cannot hold the rings (%lld bytes)", who, (long long)buffer_bytes, (long long)rings_end);
    fg_cache_t* c = new fg_cache_t();
    c->num_nodes = num_nodes;
    c->n_layers = n_layers;
    c->dtype = dtype;
    c->t_stale = t_stale;
    c->layers = n_layers ? new fg_layer[n_layers]() : nullptr;
    c->buffer_bytes = buffer_bytes;
    hipError_t e = buffer_bytes > 0 ? hipMalloc((void**)&c->buffer, (size_t)buffer_bytes) : hipSuccess;
    int64_t at = 0;
    for (int i = 0; i < n_layers && e == hipSuccess; ++i) {
        fg_layer& l = c->layers[i];
        l.capacity = capacity[i];
        l.dim = dim[i];
        at = (int64_t)fg_align_up((size_t)at, FG_RING_ALIGN);
        l.base = at;
        l.table = c->buffer + at;
        at += l.capacity * l.dim * esz;
        e = hipMalloc((void**)&l.map, (size_t)num_nodes * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&l.slot_node, (size_t)l.capacity * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&l.slot_stamp, (size_t)l.capacity * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&l.head, 32);
        if (e == hipSuccess) e = hipMalloc(&l.sel, sizeof(SelState));
    }
    if (e != hipSuccess) {
        free_layers(c);
        (void)hipGetLastError();
        FG_FAIL(e == hipErrorOutOfMemory ? FG_ERR_OOM : FG_ERR_HIP, "%s: device allocation failed: %s", who, hipGetErrorString(e));
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

extern "C" fg_status_t fg_cache_set_stabilization(fg_cache_t* cache, int64_t n_iterations) {
    if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_set_stabilization: cache is NULL");
    if (n_iterations < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_set_stabilization: n_iterations = %lld is negative", (long long)n_iterations);
    cache->stabilization = n_iterations;
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
    CacheRW c{l->map, l->slot_node, l->slot_stamp, l->head + l->head_cur, nullptr, l->head + 2, l->capacity, cache->num_nodes, iter, cache->t_stale};
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

namespace {

// Checks one layer's arguments and fills its descriptor; `ws` is the layer's share of the workspace.
fg_status_t prepare_update_layer(fg_cache_t* cache, const char* who, int32_t layer, int64_t iter, const int32_t* ids_dev,
                                 int32_t n, const uint8_t* live_dev, const uint8_t* hit_dev, const float* gnorm_dev,
                                 float p_grad, const void* h_dev, int64_t h_stride, int64_t* stats_dev, char* ws,
                                 UpdLayer* out, const int32_t* saving_dev = nullptr, int64_t max_admit = 0,
                                 const int64_t* n_dev = nullptr) {
    const fg_layer* lc;
    fg_status_t rc = layer_of(cache, layer, who, &lc);
    if (rc != FG_OK) return rc;
    const fg_layer* l = &cache->layers[layer - 1];
    if (n < 0) FG_FAIL(FG_ERR_INVALID_ARG, "%s: n = %d is negative", who, n);
    if (!(p_grad >= 0.0f && p_grad <= 1.0f)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: p_grad = %g outside [0, 1]", who, (double)p_grad);
    if (n > 0 && (!ids_dev || !hit_dev || !gnorm_dev || !h_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    const int64_t row_bytes = (int64_t)l->dim * fg_dtype_size(cache->dtype);
    if (h_stride < row_bytes) FG_FAIL(FG_ERR_SHAPE, "%s: h_stride = %lld smaller than a cache row of %lld bytes", who, (long long)h_stride, (long long)row_bytes);
    if (((uintptr_t)h_dev | (uintptr_t)h_stride) & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_dev and h_stride must be 16-byte aligned", who);
    if (iter < l->last_iter) FG_FAIL(FG_ERR_STATE, "%s: iteration %lld after %lld: the counter must not go backwards", who, (long long)iter, (long long)l->last_iter);
    if (iter < 0 || iter > INT32_MAX - 1) FG_FAIL(FG_ERR_INVALID_ARG, "%s: iteration %lld out of range", who, (long long)iter);
    if (max_admit < 0) FG_FAIL(FG_ERR_INVALID_ARG, "%s: max_admit = %lld is negative", who, (long long)max_admit);
    const UpdWs w = upd_layout(n);
    UpdLayer& u = *out;
    u.c = CacheRW{l->map, l->slot_node, l->slot_stamp, l->head + l->head_cur, l->head + (l->head_cur ^ 1), l->head + 2, l->capacity, cache->num_nodes, iter, cache->t_stale};
    u.ids = ids_dev;
    u.live = live_dev;
    u.hit = hit_dev;
    u.gnorm = gnorm_dev;
    u.stats = stats_dev;
    u.sel = (SelState*)l->sel;
    u.hdr = (UpdHeader*)(ws + w.hdr);
    u.flag = (uint8_t*)(ws + w.flag);
    u.blk = (int32_t*)(ws + w.blk);
    u.blk_sure = (int32_t*)(ws + w.blk_sure);
    u.room = (max_admit > 0 && max_admit < l->capacity) ? max_admit : l->capacity;
    u.saving = (n > 0 && u.room < n) ? saving_dev : nullptr;  // with room for every node of the layer the estimates decide nothing
    u.apos = (int32_t*)(ws + w.pos);
    u.aslot = (int32_t*)(ws + w.slot);
    u.h = (const char*)h_dev;
    u.h_stride = h_stride;
    u.table = (char*)l->table;
    u.row_bytes = row_bytes;
    u.n = n;
    u.n_dev = n_dev;
    u.p_grad = iter < cache->stabilization ? 0.0f : p_grad;  // stabilization period: nothing is admitted (k = 0)
    return FG_OK;
}

// The launches for the layers described in B (descriptors complete, first-workgroup tables not yet): `select` = the
// four (five with the access-aware ranking) launches that decide and write the cache's index, `commit` = the row copy.
fg_status_t launch_update(UpdBatch& B, hipStream_t st, bool select = true, bool commit = true) {
    B.sel_first[0] = B.scan_first[0] = 0;
    for (int i = 0; i < B.n_layers; ++i) {  // at least one workgroup per layer: it resets the statistics and writes the header
        const int64_t n = B.l[i].n > 0 ? B.l[i].n : 1;
        B.sel_first[i + 1] = B.sel_first[i] + (int)fg_ceil_div(n, SEL_CHUNK);
        B.scan_first[i + 1] = B.scan_first[i] + (int)fg_ceil_div(n, FG_SCAN_BLOCK);
    }
    const unsigned n_sel = (unsigned)B.sel_first[B.n_layers], n_scan = (unsigned)B.scan_first[B.n_layers];
    if (select) {
        hipLaunchKernelGGL(update_digit0_kernel, dim3(n_sel), dim3(SEL_THREADS), 0, st, B);
        FG_LAUNCH_CHECK("update_digit0_kernel");
        hipLaunchKernelGGL(update_digit1_kernel, dim3(n_sel), dim3(SEL_THREADS), 0, st, B);
        FG_LAUNCH_CHECK("update_digit1_kernel");
        hipLaunchKernelGGL(classify_update_kernel, dim3(n_scan), dim3(FG_SCAN_BLOCK), 0, st, B);
        FG_LAUNCH_CHECK("classify_update_kernel");
        bool ranked = false;
        for (int i = 0; i < B.n_layers; ++i) ranked |= B.l[i].saving != nullptr;
        if (ranked) {
            hipLaunchKernelGGL(rank_saving_kernel, dim3(n_scan), dim3(FG_SCAN_BLOCK), 0, st, B);
            FG_LAUNCH_CHECK("rank_saving_kernel");
        }
        hipLaunchKernelGGL(assign_slots_kernel, dim3(n_scan), dim3(FG_SCAN_BLOCK), 0, st, B);
        FG_LAUNCH_CHECK("assign_slots_kernel");
    }
    if (!commit) return FG_OK;
    fg_row_copy_batch copies;  // table[aslot[k], :] = h[apos[k], :] for the admitted rows of every layer
    copies.n = B.n_layers;
    for (int i = 0; i < B.n_layers; ++i) {
        const UpdLayer& u = B.l[i];
        const int64_t cap = u.n < u.c.capacity ? u.n : u.c.capacity;
        copies.c[i] = fg_row_copy{u.h, u.n, u.h_stride, u.apos, u.aslot, &u.hdr->n_admit, cap, u.table, u.c.capacity, u.row_bytes, u.row_bytes};
    }
    return fg_launch_row_copies(copies, st);
}

}  // namespace

extern "C" fg_status_t fg_cache_update(fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev,
                                       int32_t n, const uint8_t* live_dev, const uint8_t* hit_dev,
                                       const float* gnorm_dev, float p_grad, const void* h_dev, int64_t h_stride,
                                       int64_t* stats_dev, void* ws_dev, size_t ws_bytes, void* stream) {
    if (cache && layer >= 1 && layer <= cache->n_layers && cache->layers[layer - 1].copy_pending)
        FG_FAIL(FG_ERR_STATE, "fg_cache_update: layer %d still waits for fg_cache_update_commit", layer);
    UpdBatch B;
    B.n_layers = 1;
    fg_status_t rc = prepare_update_layer(cache, "fg_cache_update", layer, iter, ids_dev, n, live_dev, hit_dev, gnorm_dev,
                                          p_grad, h_dev, h_stride, stats_dev, (char*)ws_dev, &B.l[0]);
    if (rc != FG_OK) return rc;
    const size_t need = upd_layout(n).total;
    if (!ws_dev || ws_bytes < need) FG_FAIL(FG_ERR_SHAPE, "fg_cache_update: workspace of %zu bytes given, %zu needed", ws_bytes, need);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_update: workspace must be 16-byte aligned");
    fg_clear_error();
    rc = launch_update(B, (hipStream_t)stream);
    if (rc != FG_OK) return rc;
    fg_layer* l = &cache->layers[layer - 1];
    l->last_iter = iter;
    l->head_cur ^= 1;  // the advanced header written by assign_slots is the current one from here on
    return FG_OK;
}

namespace {

// phase 0: the whole update; 1: selection and index only; 2: the row copy of a selection made by phase 1 with the same
// descriptors and workspace (the ring headers have been swapped by then, so the descriptors are rebuilt without them)
fg_status_t update_all(const char* who, int phase, fg_cache_t* cache, int64_t iter, float p_grad, int32_t n_layers,
                       const fg_update_layer_t* layers, void* ws_dev, size_t ws_bytes, void* stream) {
    if (n_layers < 0 || n_layers > FG_MAX_UPD_LAYERS) FG_FAIL(FG_ERR_INVALID_ARG, "%s: n_layers = %d outside 0..%d", who, n_layers, FG_MAX_UPD_LAYERS);
    if (n_layers > 0 && !layers) FG_FAIL(FG_ERR_INVALID_ARG, "%s: layers is NULL", who);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: workspace must be 16-byte aligned", who);
    if (phase == 2 && n_layers > 0) {
        if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "%s: cache is NULL", who);
        for (int i = 0; i < n_layers; ++i) {
            const int32_t layer = layers[i].layer;
            if (layer < 1 || layer > cache->n_layers) FG_FAIL(FG_ERR_INVALID_ARG, "%s: layer %d outside 1..%d", who, layer, cache->n_layers);
            if (cache->layers[layer - 1].last_iter != iter || !cache->layers[layer - 1].copy_pending)
                FG_FAIL(FG_ERR_STATE, "%s: layer %d has no selection of iteration %lld waiting for its rows", who, layer, (long long)iter);
        }
    }
    UpdBatch B;
    B.n_layers = n_layers;
    size_t off = 0;
    for (int i = 0; i < n_layers; ++i) {
        for (int k = 0; k < i; ++k)
            if (layers[k].layer == layers[i].layer) FG_FAIL(FG_ERR_INVALID_ARG, "%s: layer %d is listed twice", who, layers[i].layer);
        const fg_update_layer_t& a = layers[i];
        if (phase != 2 && cache && a.layer >= 1 && a.layer <= cache->n_layers && cache->layers[a.layer - 1].copy_pending)
            FG_FAIL(FG_ERR_STATE, "%s: layer %d still waits for fg_cache_update_commit", who, a.layer);
        fg_status_t rc = prepare_update_layer(cache, who, a.layer, phase == 2 ? cache->layers[a.layer - 1].last_iter : iter, a.ids_dev, a.n,
                                              a.live_dev, a.hit_dev, a.gnorm_dev, p_grad, a.h_dev, a.h_stride, a.stats_dev,
                                              (char*)ws_dev + off, &B.l[i], a.saving_dev, a.max_admit, a.n_dev);
        if (rc != FG_OK) return rc;
        off += upd_layout(a.n).total;
    }
    if (n_layers > 0 && (!ws_dev || ws_bytes < off)) FG_FAIL(FG_ERR_SHAPE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes, off);
    fg_clear_error();
    if (n_layers == 0) return FG_OK;
    fg_status_t rc = launch_update(B, (hipStream_t)stream, phase != 2, phase != 1);
    if (rc != FG_OK) return rc;
    for (int i = 0; i < n_layers; ++i) {
        fg_layer* l = &cache->layers[layers[i].layer - 1];
        if (phase != 2) {
            l->last_iter = iter;
            l->head_cur ^= 1;
        }
        l->copy_pending = phase == 1;
    }
    return FG_OK;
}

}  // namespace

extern "C" fg_status_t fg_cache_update_all(fg_cache_t* cache, int64_t iter, float p_grad, int32_t n_layers,
                                           const fg_update_layer_t* layers, void* ws_dev, size_t ws_bytes, void* stream) {
    return update_all("fg_cache_update_all", 0, cache, iter, p_grad, n_layers, layers, ws_dev, ws_bytes, stream);
}

extern "C" fg_status_t fg_cache_update_select(fg_cache_t* cache, int64_t iter, float p_grad, int32_t n_layers,
                                              const fg_update_layer_t* layers, void* ws_dev, size_t ws_bytes, void* stream) {
    return update_all("fg_cache_update_select", 1, cache, iter, p_grad, n_layers, layers, ws_dev, ws_bytes, stream);
}

extern "C" fg_status_t fg_cache_update_commit(fg_cache_t* cache, int64_t iter, int32_t n_layers, const fg_update_layer_t* layers,
                                              void* ws_dev, size_t ws_bytes, void* stream) {
    return update_all("fg_cache_update_commit", 2, cache, iter, 0.0f, n_layers, layers, ws_dev, ws_bytes, stream);
}

// ---- estimate of saved accesses (input of the access-aware admission) -------------------------------------------

namespace {

constexpr int EST_THREADS = 256;

// One thread per row of a pruned block: 1 for a node served from the cache; otherwise what its own row of the layer
// below and each remaining neighbour read (1 each when the layer below is the input layer). Saturates at 2047.
__global__ __launch_bounds__(EST_THREADS) void access_estimate_kernel(const int32_t* __restrict__ row_start,
                                                                      const int32_t* __restrict__ row_end,
                                                                      const int32_t* __restrict__ col, int64_t nnz, int n,
                                                                      const uint8_t* __restrict__ hit,
                                                                      const int32_t* __restrict__ below, int n_src,
                                                                      int32_t* __restrict__ out) {
    const int j = blockIdx.x * EST_THREADS + threadIdx.x;
    if (j >= n) return;
    if (hit && hit[j]) {
        out[j] = 1;
        return;
    }
    int64_t b = row_start[j], e = row_end[j];
    if (b < 0) b = 0;
    if (e > nnz) e = nnz;
    int64_t total = below ? (j < n_src ? clamp_saving(below[j]) : 0) : 1;
    for (int64_t c = b; c < e; ++c) {
        if (below) {
            const int32_t u = col[c];
            if (u >= 0 && u < n_src) total += clamp_saving(below[u]);
        } else {
            total += 1;
        }
    }
    out[j] = total > 2047 ? 2047 : (int32_t)total;
}

}  // namespace

extern "C" fg_status_t fg_access_estimate(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                                          int64_t nnz, int32_t n, const uint8_t* hit_dev, const int32_t* below_dev,
                                          int32_t n_src, int32_t* out_dev, void* stream) {
    if (n < 0 || nnz < 0 || n_src < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_access_estimate: negative size");
    if (n > 0 && (!row_start_dev || !row_end_dev || !out_dev || (nnz > 0 && !col_dev)))
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_access_estimate: NULL pointer");
    if (below_dev && n_src < n) FG_FAIL(FG_ERR_SHAPE, "fg_access_estimate: the layer below has %d nodes, fewer than this layer's %d", n_src, n);
    fg_clear_error();
    if (n == 0) return FG_OK;
    hipLaunchKernelGGL(access_estimate_kernel, dim3((unsigned)fg_ceil_div(n, EST_THREADS)), dim3(EST_THREADS), 0, (hipStream_t)stream,
                       row_start_dev, row_end_dev, col_dev, nnz, n, hit_dev, below_dev, n_src, out_dev);
    FG_LAUNCH_CHECK("access_estimate_kernel");
    return FG_OK;
}

fg_status_t fg_build_fetch_batch(const char* who, const fg_cache_t* cache, int32_t n_layers, const fg_fetch_layer_t* layers,
                                 fg_row_copy_batch* out) {
    if (n_layers < 0 || n_layers > FG_MAX_COPIES) FG_FAIL(FG_ERR_INVALID_ARG, "%s: n_layers = %d outside 0..%d", who, n_layers, FG_MAX_COPIES);
    if (n_layers > 0 && !layers) FG_FAIL(FG_ERR_INVALID_ARG, "%s: layers is NULL", who);
    out->n = n_layers;
    for (int i = 0; i < n_layers; ++i) {
        const fg_fetch_layer_t& a = layers[i];
        const fg_layer* l;
        fg_status_t rc = layer_of(cache, a.layer, who, &l);
        if (rc != FG_OK) return rc;
        if (a.max_hits < 0 || a.h_rows < 0) FG_FAIL(FG_ERR_INVALID_ARG, "%s: negative size for layer %d", who, a.layer);
        if (a.max_hits > 0 && (!a.hit_slot_dev || !a.hit_pos_dev || !a.h_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer for layer %d", who, a.layer);
        const int64_t row_bytes = (int64_t)l->dim * fg_dtype_size(cache->dtype);
        if (a.h_stride < row_bytes)
            FG_FAIL(FG_ERR_SHAPE, "%s: h_stride = %lld smaller than a cache row of %lld bytes", who, (long long)a.h_stride, (long long)row_bytes);
        if (((uintptr_t)a.h_dev | (uintptr_t)a.h_stride) & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_dev and h_stride must be 16-byte aligned", who);
        out->c[i] = fg_row_copy{(const char*)l->table, l->capacity, row_bytes, a.hit_slot_dev, a.hit_pos_dev, a.n_hit_dev, a.max_hits,
                                (char*)a.h_dev, a.h_rows, a.h_stride, row_bytes};
    }
    return FG_OK;
}

extern "C" fg_status_t fg_cache_fetch_all(const fg_cache_t* cache, int32_t n_layers, const fg_fetch_layer_t* layers,
                                          void* stream) {
    fg_row_copy_batch copies;
    fg_status_t rc = fg_build_fetch_batch("fg_cache_fetch_all", cache, n_layers, layers, &copies);
    if (rc != FG_OK) return rc;
    fg_clear_error();
    return fg_launch_row_copies(copies, (hipStream_t)stream);
}

// ---- feature side of the shared buffer (Section 4.2) ---------------------------------------------------------
//
// Before training the raw feature rows of a caller-ordered hot list are copied to the right end of the buffer,
// the hottest farthest from the rings. Nothing ever moves or invalidates them explicitly: a row counts as lost
// once a ring has written over any of its bytes, which a reader decides from the rings' `used` counters
// (fg_feature_rank). The loader variants consult the node -> rank array first and read a surviving row from HBM
// instead of the feature table.

fg_feat_side fg_feature_side(const fg_cache_t* cache) {
    fg_feat_side F = {};
    if (!cache || cache->n_feat <= 0 || !cache->feat_rank) return F;
    F.rank = cache->feat_rank;
    F.end = cache->buffer + cache->buffer_bytes;
    F.row_bytes = cache->feat_row_bytes;
    F.n_rows = cache->n_feat;
    F.buffer_bytes = cache->buffer_bytes;
    F.n_rings = cache->n_layers;
    for (int i = 0; i < cache->n_layers && i < FG_MAX_RINGS; ++i) {
        const fg_layer& l = cache->layers[i];
        F.ring_lo[i] = l.base;
        F.ring_row[i] = (int64_t)l.dim * fg_dtype_size(cache->dtype);
        F.ring_used[i] = l.head + 2;
    }
    return F;
}

namespace {

constexpr int FEAT_THREADS = 256;

// One wavefront per rank: rank[hot[r]] = r and the node's table row goes to end - (r+1)*row_bytes.
__global__ __launch_bounds__(FEAT_THREADS) void place_features_kernel(const int32_t* __restrict__ hot, int64_t n_hot,
                                                                      const char* __restrict__ table, int64_t table_rows,
                                                                      int64_t src_stride, int64_t row_bytes,
                                                                      int32_t* __restrict__ rank, int64_t num_nodes,
                                                                      char* __restrict__ end) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & 63;
    const int chunks = (int)(row_bytes >> 4);
    const int64_t n_waves = ((int64_t)gridDim.x * FEAT_THREADS) >> 6;
    for (int64_t r = ((int64_t)blockIdx.x * FEAT_THREADS + threadIdx.x) >> 6; r < n_hot; r += n_waves) {
        const int32_t v = hot[r];
        if (v < 0 || v >= num_nodes || v >= table_rows) continue;  // the rank stays unused
        if (lane == 0) rank[v] = (int32_t)r;
        const u32x4* src = (const u32x4*)(table + (int64_t)v * src_stride);
        u32x4* dst = (u32x4*)(end - (r + 1) * row_bytes);
        for (int c = lane; c < chunks; c += 64) dst[c] = __builtin_nontemporal_load(src + c);
    }
}

__global__ __launch_bounds__(FEAT_THREADS) void feature_lookup_kernel(fg_feat_side F, int64_t num_nodes,
                                                                      const int32_t* __restrict__ ids,
                                                                      const int64_t* __restrict__ count_dev, int64_t max_count,
                                                                      int32_t* __restrict__ rank_out,
                                                                      unsigned long long* __restrict__ n_found) {
    int64_t count = count_dev ? *count_dev : max_count;
    if (count > max_count) count = max_count;
    int found = 0;
    for (int64_t k = (int64_t)blockIdx.x * FEAT_THREADS + threadIdx.x; k < count; k += (int64_t)gridDim.x * FEAT_THREADS) {
        const int32_t v = ids[k];
        const int32_t r = (F.rank && v >= 0 && v < num_nodes) ? fg_feature_rank(F, v) : -1;
        if (rank_out) rank_out[k] = r;
        found += r >= 0;
    }
    if (n_found) {
        __shared__ int red[FEAT_THREADS / 64];
        int w = found;
        for (int off = 32; off > 0; off >>= 1) w += __shfl_down(w, off, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
        __syncthreads();
        if (threadIdx.x == 0) {
            int s = 0;
            for (int i = 0; i < FEAT_THREADS / 64; ++i) s += red[i];
            if (s) atomicAdd(n_found, (unsigned long long)s);
        }
    }
}

}  // namespace

extern "C" fg_status_t fg_cache_fill_features(fg_cache_t* cache, const int32_t* hot_ids_dev, int64_t n_hot, const void* table,
                                              int64_t table_rows, int64_t src_stride, int64_t row_bytes, void* stream) {
    if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_fill_features: cache is NULL");
    if (n_hot < 0 || table_rows < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_fill_features: negative size");
    if (n_hot > INT32_MAX) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_fill_features: n_hot = %lld exceeds 2^31-1", (long long)n_hot);
    if (n_hot > 0 && (!hot_ids_dev || !table)) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_fill_features: hot_ids_dev and table are required");
    if (row_bytes <= 0 || row_bytes % 16) FG_FAIL(FG_ERR_SHAPE, "fg_cache_fill_features: row_bytes = %lld must be a positive multiple of 16", (long long)row_bytes);
    if (src_stride < row_bytes) FG_FAIL(FG_ERR_SHAPE, "fg_cache_fill_features: src_stride = %lld smaller than a row of %lld bytes", (long long)src_stride, (long long)row_bytes);
    if (((uintptr_t)table | (uintptr_t)src_stride) & 15) FG_FAIL(FG_ERR_INVALID_ARG, "fg_cache_fill_features: table and src_stride must be 16-byte aligned");
    if (cache->n_layers > FG_MAX_RINGS) FG_FAIL(FG_ERR_SHAPE, "fg_cache_fill_features: at most %d cached layers share a buffer with features", FG_MAX_RINGS);
    if (cache->buffer_bytes % 16) FG_FAIL(FG_ERR_STATE, "fg_cache_fill_features: the buffer size is not a multiple of 16");
    if (n_hot > cache->buffer_bytes / row_bytes)
        FG_FAIL(FG_ERR_SHAPE, "fg_cache_fill_features: %lld rows of %lld bytes do not fit into the buffer of %lld bytes", (long long)n_hot,
                (long long)row_bytes, (long long)cache->buffer_bytes);
    for (int i = 0; i < cache->n_layers; ++i)
        if (cache->layers[i].last_iter != INT64_MIN)
            FG_FAIL(FG_ERR_STATE, "fg_cache_fill_features: layer %d has been updated; features are placed into an empty cache (after create or clear)", i + 1);
    hipStream_t st = (hipStream_t)stream;
    if (!cache->feat_rank) {
        hipError_t e = hipMalloc((void**)&cache->feat_rank, (size_t)cache->num_nodes * 4);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            cache->feat_rank = nullptr;
            FG_FAIL(e == hipErrorOutOfMemory ? FG_ERR_OOM : FG_ERR_HIP, "fg_cache_fill_features: allocating the rank array failed: %s", hipGetErrorString(e));
        }
    }
    fg_clear_error();
    fg_status_t rc = fg_launch_fill_i32(cache->feat_rank, cache->num_nodes, -1, st);
    if (rc != FG_OK) return rc;
    cache->n_feat = n_hot;
    cache->feat_row_bytes = n_hot > 0 ? row_bytes : 0;
    if (n_hot == 0) return FG_OK;
    int64_t blocks = fg_ceil_div(n_hot, FEAT_THREADS / 64);
    if (blocks > 256 * 8) blocks = 256 * 8;
    hipLaunchKernelGGL(place_features_kernel, dim3((unsigned)blocks), dim3(FEAT_THREADS), 0, st, hot_ids_dev, n_hot, (const char*)table,
                       table_rows, src_stride, row_bytes, cache->feat_rank, cache->num_nodes, cache->buffer + cache->buffer_bytes);
    FG_LAUNCH_CHECK("place_features_kernel");
    return FG_OK;
}

extern "C" fg_status_t fg_feature_lookup(const fg_cache_t* cache, const int32_t* ids_dev, const int64_t* count_dev, int64_t max_count,
                                         int32_t* rank_out_dev, int64_t* n_found_dev, void* stream) {
    if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "fg_feature_lookup: cache is NULL");
    if (max_count < 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_feature_lookup: max_count = %lld is negative", (long long)max_count);
    if (max_count > 0 && !ids_dev) FG_FAIL(FG_ERR_INVALID_ARG, "fg_feature_lookup: ids_dev is NULL");
    fg_clear_error();
    hipStream_t st = (hipStream_t)stream;
    if (n_found_dev) {
        fg_status_t rc = fg_launch_fill_i32((int32_t*)n_found_dev, 2, 0, st);
        if (rc != FG_OK) return rc;
    }
    if (max_count == 0) return FG_OK;
    int64_t blocks = fg_ceil_div(max_count, FEAT_THREADS);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(feature_lookup_kernel, dim3((unsigned)blocks), dim3(FEAT_THREADS), 0, st, fg_feature_side(cache), cache->num_nodes,
                       ids_dev, count_dev, max_count, rank_out_dev, (unsigned long long*)n_found_dev);
    FG_LAUNCH_CHECK("feature_lookup_kernel");
    return FG_OK;
}

extern "C" const void* fg_cache_buffer(const fg_cache_t* cache, int64_t* buffer_bytes_out) {
    if (buffer_bytes_out) *buffer_bytes_out = cache ? cache->buffer_bytes : 0;
    return cache ? cache->buffer : nullptr;
}

extern "C" int64_t fg_cache_feature_rows(const fg_cache_t* cache) { return cache ? cache->n_feat : 0; }

extern "C" int64_t fg_cache_ring_offset(const fg_cache_t* cache, int32_t layer) {
    const fg_layer* l;
    if (layer_of(cache, layer, "fg_cache_ring_offset", &l) != FG_OK) return -1;
    return l->base;
}
