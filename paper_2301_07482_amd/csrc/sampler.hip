// Neighbour sampling of one block on the device (the uniform fan-out sampling of Section 7.1, which the paper runs on
// CPU threads, Section 5): from the nodes of layer l to the block (start, end, columns) and the node list of layer l-1,
// over an in-neighbour CSR held in device-visible memory.
//
// Per node v with degree d and fan-out f: slots 0..d-1 when d <= f; otherwise the row is cut into f disjoint strata
// with integer bounds, stratum j = [floor(j d / f), floor((j + 1) d / f)), draw j takes the slot at offset
// floor(u_j * width_j) of stratum j, and the f slots are moved round the row by a common offset floor(u_f * d) modulo d
// (f distinct slots, every slot of the row with probability f / d); u_j from the counter-based SplitMix64 generator
// keyed by (mini-batch key, layer, v, j); the neighbours at those slots in the order of j, without v and without repeats. The layer
// below is the layer's own nodes followed by the new neighbours in order of first occurrence; columns are positions in
// that list. Everything is a pure function of the inputs: no atomics decide an order, so the result is the same in
// every run.
//
// Launches (sizes from the host-side bound max_rows, the exact count is read on the device):
//   0. clear the hash table
//   1. draw      32 lanes per row: slot, neighbour, repeats removed by comparing within the row; per-row and
//                per-workgroup counts; the layer's own nodes go to the head of the list below and into the table
//   2. compact   rows back to back (start/end), candidates in row order; every candidate enters the table with its
//                order number n + k; the table keeps the smallest order number per node
//   3. resolve   per candidate: the smallest order number of its node; it is a first occurrence iff that is its own
//   4. number    first occurrences are ranked in candidate order and appended to the list below
//   5. columns   position of every candidate's node in the list below
#include "common.h"
#include "scan.h"

namespace {

constexpr int SMP_THREADS = 1024;
constexpr int SMP_LANES = 32;                           // lanes per row: the largest fan-out
constexpr int SMP_ROWS = SMP_THREADS / SMP_LANES;       // rows per workgroup
constexpr unsigned long long SMP_EMPTY = ~0ull;

__host__ __device__ inline uint64_t smp_mix(uint64_t x) {
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}
__host__ __device__ inline uint64_t smp_word(uint64_t key, uint64_t counter) {
    return smp_mix(key + (counter + 1ull) * 0x9E3779B97F4A7C15ull);
}

struct SmpArgs {
    const int64_t* indptr;
    const int32_t* indices;
    int64_t num_nodes, num_edges;
    const int32_t* ids;
    const int64_t* n_dev;
    int64_t max_rows;
    int32_t fanout;
    uint64_t key_l;
    int32_t* row_start;
    int32_t* row_end;
    int32_t* col;
    int32_t* col_ids;     // candidates in row order (a workspace array when the caller wants no ids)
    int32_t* below;
    int64_t max_below;
    int64_t* counts;      // [0] nodes of the layer below, [1] edges
    int32_t* nbuf;        // [max_rows * fanout] raw candidates, -1 = none
    int32_t* cnt;         // [max_rows]
    int32_t* blk_rows;    // candidates per workgroup of launch 1
    int32_t* first;       // [max_rows * fanout] smallest order number of the candidate's node
    int32_t* rank;        // [max_rows * fanout] rank among the first occurrences
    int32_t* blk_new;     // first occurrences per workgroup of launch 3
    unsigned long long* table;
    uint32_t mask;        // table entries - 1 (a power of two)
    int shift;            // 32 - log2(entries)
};

__device__ __forceinline__ int64_t smp_rows(const SmpArgs& A) {
    int64_t n = A.n_dev ? *A.n_dev : A.max_rows;
    if (n < 0) n = 0;
    return n < A.max_rows ? n : A.max_rows;
}

__device__ __forceinline__ uint32_t smp_hash(const SmpArgs& A, int32_t node) { return ((uint32_t)node * 0x9E3779B1u) >> A.shift; }

// Keeps the smallest order number seen for `node`. An entry's node never changes once it is set.
__device__ __forceinline__ void smp_insert(const SmpArgs& A, int32_t node, uint32_t order) {
    const unsigned long long mine = ((unsigned long long)(uint32_t)node << 32) | order;
    uint32_t h = smp_hash(A, node);
    for (uint32_t probe = 0; probe <= A.mask; ++probe) {
        // most nodes occur once, so the slot is usually empty: one operation instead of a load followed by one
        const unsigned long long cur = atomicCAS(&A.table[h], SMP_EMPTY, mine);
        if (cur == SMP_EMPTY) return;
        if ((uint32_t)(cur >> 32) == (uint32_t)node) {
            atomicMin(&A.table[h], mine);
            return;
        }
        h = (h + 1) & A.mask;
    }
}

__device__ __forceinline__ int64_t smp_lookup(const SmpArgs& A, int32_t node) {
    uint32_t h = smp_hash(A, node);
    for (uint32_t probe = 0; probe <= A.mask; ++probe) {
        const unsigned long long cur = A.table[h];
        if (cur == SMP_EMPTY) return -1;
        if ((uint32_t)(cur >> 32) == (uint32_t)node) return (int64_t)(uint32_t)cur;
        h = (h + 1) & A.mask;
    }
    return -1;
}

__global__ __launch_bounds__(SMP_THREADS) void sample_draw_kernel(SmpArgs A) {
    __shared__ int s_cnt[SMP_ROWS];
    const int64_t n = smp_rows(A);
    const int g = threadIdx.x / SMP_LANES, j = threadIdx.x % SMP_LANES;
    const int64_t row = (int64_t)blockIdx.x * SMP_ROWS + g;
    const int f = A.fanout;
    int32_t v = -1, nb = -1;
    bool ok = false;
    if (row < n) {
        v = A.ids[row];
        if (v >= 0 && v < A.num_nodes) {
            const int64_t lo = A.indptr[v], d = A.indptr[(int64_t)v + 1] - lo;
            if (j < f && j < d) {
                int64_t slot = j;
                if (d > f) {
                    const uint64_t kv = smp_word(A.key_l, (uint64_t)v);
                    const double scale = 1.0 / 9007199254740992.0;
                    const double u = (double)(smp_word(kv, (uint64_t)j) >> 11) * scale;
                    const double ut = (double)(smp_word(kv, (uint64_t)f) >> 11) * scale;
                    const int64_t first = ((int64_t)j * d) / f, width = ((int64_t)(j + 1) * d) / f - first;
                    int64_t inside = (int64_t)(u * (double)width);
                    if (inside > width - 1) inside = width - 1;
                    int64_t turn = (int64_t)(ut * (double)d);
                    if (turn > d - 1) turn = d - 1;
                    slot = (first + inside + turn) % d;
                }
                const int64_t at = lo + slot;
                if (at >= 0 && at < A.num_edges) {
                    nb = A.indices[at];
                    ok = nb != v && nb >= 0 && nb < A.num_nodes;
                }
            }
        }
    }
    // an earlier slot of the row with the same neighbour removes this one (self loops never count as earlier)
    bool keep = ok;
    for (int b = 0; b < f - 1; ++b) {
        const int32_t other = __shfl(nb, b, SMP_LANES);
        const bool other_ok = __shfl((int)ok, b, SMP_LANES) != 0;
        if (b < j && other_ok && other == nb) keep = false;
    }
    const unsigned long long kept = __ballot(keep);
    const uint32_t mine = (uint32_t)(kept >> (32 * ((threadIdx.x >> 5) & 1)));
    if (row < A.max_rows) {
        if (j < f) A.nbuf[row * f + j] = keep ? nb : -1;
        if (j == 0) {
            A.cnt[row] = row < n ? __popc(mine) : 0;
            if (row < n) {
                if (row < A.max_below) A.below[row] = v;
                if (v >= 0) smp_insert(A, v, (uint32_t)row);
            }
        }
    }
    if (j == 0) s_cnt[g] = row < n ? __popc(mine) : 0;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int q = 0; q < SMP_ROWS; ++q) t += s_cnt[q];
        A.blk_rows[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(SMP_THREADS) void sample_compact_kernel(SmpArgs A) {
    __shared__ long long red[16];
    __shared__ int s_cnt[SMP_ROWS];
    const int64_t n = smp_rows(A);
    const int g = threadIdx.x / SMP_LANES, j = threadIdx.x % SMP_LANES;
    const int64_t row = (int64_t)blockIdx.x * SMP_ROWS + g;
    const int f = A.fanout;
    long long before = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += SMP_THREADS) before += A.blk_rows[b];
    before = fg_block_sum(before, red);
    const int c = row < A.max_rows ? A.cnt[row] : 0;
    if (j == 0) s_cnt[g] = c;
    __syncthreads();
    long long first = before;
    for (int q = 0; q < g; ++q) first += s_cnt[q];
    const int32_t nb = (row < A.max_rows && j < f) ? A.nbuf[row * f + j] : -1;
    const bool keep = nb >= 0;
    const unsigned long long kept = __ballot(keep);
    const uint32_t mine = (uint32_t)(kept >> (32 * ((threadIdx.x >> 5) & 1)));
    const int r = __popc(mine & ((1u << j) - 1u));
    if (row < A.max_rows && j == 0) {
        A.row_start[row] = (int32_t)first;
        A.row_end[row] = (int32_t)(first + c);
    }
    if (keep) {
        const long long k = first + r;
        A.col_ids[k] = nb;
        smp_insert(A, nb, (uint32_t)(n + k));
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        long long all = before;
        for (int q = 0; q < SMP_ROWS; ++q) all += s_cnt[q];
        A.counts[1] = all;
    }
}

// One thread per candidate. The number of candidates is the end of the last row.
__device__ __forceinline__ int64_t smp_edges(const SmpArgs& A, int64_t n) { return n > 0 ? (int64_t)A.row_end[n - 1] : 0; }

__global__ __launch_bounds__(FG_SCAN_BLOCK) void sample_resolve_kernel(SmpArgs A) {
    const int64_t n = smp_rows(A);
    const int64_t nnz = smp_edges(A, n);
    const int64_t k = (int64_t)blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    bool is_first = false;
    if (k < nnz) {
        const int64_t m = smp_lookup(A, A.col_ids[k]);
        A.first[k] = (int32_t)m;
        is_first = m == n + k;
    }
    const int t = __syncthreads_count(is_first);
    if (threadIdx.x == 0) A.blk_new[blockIdx.x] = t;
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void sample_number_kernel(SmpArgs A) {
    __shared__ long long red[16];
    __shared__ int sc[17];
    const int64_t n = smp_rows(A);
    const int64_t nnz = smp_edges(A, n);
    const int64_t k = (int64_t)blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    long long before = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += FG_SCAN_BLOCK) before += A.blk_new[b];
    before = fg_block_sum(before, red);
    const bool is_first = k < nnz && (int64_t)A.first[k] == n + k;
    int total;
    const long long r = before + fg_block_rank(is_first, total, sc);
    if (is_first) {
        A.rank[k] = (int32_t)r;
        if (n + r < A.max_below) A.below[n + r] = A.col_ids[k];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) A.counts[0] = n + before + total;
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void sample_columns_kernel(SmpArgs A) {
    const int64_t n = smp_rows(A);
    const int64_t nnz = smp_edges(A, n);
    const int64_t k = (int64_t)blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    if (k >= nnz) return;
    const int64_t m = A.first[k];
    A.col[k] = m < n ? (int32_t)m : (int32_t)(n + A.rank[m - n]);
}

struct SmpWs {
    size_t nbuf, cnt, blk_rows, first, rank, blk_new, cand, table, total;
    uint32_t entries;
};
SmpWs smp_layout(int64_t max_rows, int32_t fanout) {
    SmpWs w;
    const size_t rows = (size_t)(max_rows > 0 ? max_rows : 1), cands = rows * (size_t)fanout;
    size_t at = 0;
    auto take = [&](size_t bytes) {
        const size_t here = at;
        at += fg_align_up(bytes, 256);
        return here;
    };
    w.nbuf = take(cands * 4);
    w.cnt = take(rows * 4);
    w.blk_rows = take((size_t)fg_ceil_div((int64_t)rows, SMP_ROWS) * 4);
    w.first = take(cands * 4);
    w.rank = take(cands * 4);
    w.blk_new = take((size_t)fg_ceil_div((int64_t)cands, FG_SCAN_BLOCK) * 4);
    w.cand = take(cands * 4);
    uint32_t entries = 1024;
    while ((size_t)entries < 2 * (rows + cands) && entries < (1u << 31)) entries <<= 1;
    w.entries = entries;
    w.table = take((size_t)entries * 8);
    w.total = at;
    return w;
}

}  // namespace

extern "C" size_t fg_sample_block_workspace_bytes(int64_t max_rows, int32_t fanout) {
    if (max_rows < 0 || fanout < 1 || fanout > SMP_LANES || max_rows > (int64_t)INT32_MAX / SMP_LANES) return 0;
    return smp_layout(max_rows, fanout).total;
}

extern "C" fg_status_t fg_sample_block(const int64_t* indptr_dev, const int32_t* indices_dev, int64_t num_nodes, int64_t num_edges,
                                       const int32_t* ids_dev, const int64_t* n_dev, int64_t max_rows, int32_t fanout, uint64_t key,
                                       int32_t layer, int32_t* row_start_dev, int32_t* row_end_dev, int32_t* col_dev,
                                       int32_t* col_ids_dev, int32_t* ids_below_dev, int64_t max_below, int64_t* counts_dev,
                                       void* ws_dev, size_t ws_bytes, void* stream) {
    const char* who = "fg_sample_block";
    if (max_rows < 0 || num_nodes <= 0 || num_edges < 0 || max_below < 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: bad size (max_rows %lld, num_nodes %lld, num_edges %lld, max_below %lld)", who,
                (long long)max_rows, (long long)num_nodes, (long long)num_edges, (long long)max_below);
    if (num_nodes > INT32_MAX) FG_FAIL(FG_ERR_INVALID_ARG, "%s: node ids are 32-bit", who);
    if (fanout < 1 || fanout > SMP_LANES) FG_FAIL(FG_ERR_INVALID_ARG, "%s: fanout = %d outside 1..%d", who, fanout, SMP_LANES);
    if (max_rows > (int64_t)INT32_MAX / SMP_LANES) FG_FAIL(FG_ERR_SHAPE, "%s: max_rows = %lld: edge numbers are 32-bit", who, (long long)max_rows);
    if (layer < 1) FG_FAIL(FG_ERR_INVALID_ARG, "%s: layer = %d, blocks are numbered from 1", who, layer);
    if (!counts_dev) FG_FAIL(FG_ERR_INVALID_ARG, "%s: counts_dev is NULL", who);
    if (max_rows > 0 && (!indptr_dev || !ids_dev || !row_start_dev || !row_end_dev || !col_dev || !ids_below_dev || (num_edges > 0 && !indices_dev)))
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (max_below < max_rows) FG_FAIL(FG_ERR_SHAPE, "%s: max_below = %lld smaller than max_rows = %lld (the layer below starts with this layer)", who, (long long)max_below, (long long)max_rows);
    const SmpWs w = smp_layout(max_rows, fanout);
    if (max_rows > 0 && (!ws_dev || ws_bytes < w.total)) FG_FAIL(FG_ERR_SHAPE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes, w.total);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: workspace must be 16-byte aligned", who);
    fg_clear_error();
    hipStream_t st = (hipStream_t)stream;
    if (max_rows == 0) {
        fg_status_t rc = fg_launch_fill_i32((int32_t*)counts_dev, 4, 0, st);
        return rc;
    }
    char* ws = (char*)ws_dev;
    SmpArgs A;
    A.indptr = indptr_dev;
    A.indices = indices_dev;
    A.num_nodes = num_nodes;
    A.num_edges = num_edges;
    A.ids = ids_dev;
    A.n_dev = n_dev;
    A.max_rows = max_rows;
    A.fanout = fanout;
    A.key_l = smp_word(smp_mix(key), (uint64_t)layer);
    A.row_start = row_start_dev;
    A.row_end = row_end_dev;
    A.col = col_dev;
    A.col_ids = col_ids_dev ? col_ids_dev : (int32_t*)(ws + w.cand);
    A.below = ids_below_dev;
    A.max_below = max_below;
    A.counts = counts_dev;
    A.nbuf = (int32_t*)(ws + w.nbuf);
    A.cnt = (int32_t*)(ws + w.cnt);
    A.blk_rows = (int32_t*)(ws + w.blk_rows);
    A.first = (int32_t*)(ws + w.first);
    A.rank = (int32_t*)(ws + w.rank);
    A.blk_new = (int32_t*)(ws + w.blk_new);
    A.table = (unsigned long long*)(ws + w.table);
    A.mask = w.entries - 1;
    int lg = 0;
    while ((1u << lg) < w.entries) ++lg;
    A.shift = 32 - lg;
    fg_status_t rc = fg_launch_fill_i32((int32_t*)A.table, (int64_t)w.entries * 2, -1, st);
    if (rc != FG_OK) return rc;
    const unsigned row_blocks = (unsigned)fg_ceil_div(max_rows, SMP_ROWS);
    const unsigned cand_blocks = (unsigned)fg_ceil_div(max_rows * fanout, FG_SCAN_BLOCK);
    hipLaunchKernelGGL(sample_draw_kernel, dim3(row_blocks), dim3(SMP_THREADS), 0, st, A);
    FG_LAUNCH_CHECK("sample_draw_kernel");
    hipLaunchKernelGGL(sample_compact_kernel, dim3(row_blocks), dim3(SMP_THREADS), 0, st, A);
    FG_LAUNCH_CHECK("sample_compact_kernel");
    hipLaunchKernelGGL(sample_resolve_kernel, dim3(cand_blocks), dim3(FG_SCAN_BLOCK), 0, st, A);
    FG_LAUNCH_CHECK("sample_resolve_kernel");
    hipLaunchKernelGGL(sample_number_kernel, dim3(cand_blocks), dim3(FG_SCAN_BLOCK), 0, st, A);
    FG_LAUNCH_CHECK("sample_number_kernel");
    hipLaunchKernelGGL(sample_columns_kernel, dim3(cand_blocks), dim3(FG_SCAN_BLOCK), 0, st, A);
    FG_LAUNCH_CHECK("sample_columns_kernel");
    return FG_OK;
}

// ---- transpose of a sampled block (what the backward pass walks) ---------------------------------------------------
//
// For every position j of the layer below: the rows that sampled it, ascending, back to back. Launches: clear the
// counters; count the edges per source; sum the counters per workgroup; exclusive scan (t_start, t_end); every edge
// takes the next free place of its source's list (the order of arrival is arbitrary); every list is sorted (lists are
// short: a source is sampled by a handful of rows), which makes the result independent of that order.
namespace {

constexpr int TR_THREADS = 256;

struct TrArgs {
    const int32_t* row_start;
    const int32_t* row_end;
    const int32_t* col;
    const int64_t* n_dev;
    int64_t max_rows;
    const int64_t* n_src_dev;
    int64_t max_src;
    int64_t max_nnz;
    int32_t* t_start;
    int32_t* t_end;
    int32_t* t_row;
    int32_t* cnt;   // [max_src] edges per source, then the next free place of its list
    int32_t* blk;   // per workgroup of the scan
};

__device__ __forceinline__ int64_t tr_count(const int64_t* dev, int64_t bound) {
    int64_t n = dev ? *dev : bound;
    if (n < 0) n = 0;
    return n < bound ? n : bound;
}

// f(row, source) for every edge of row `i` that names a valid source
template <typename F>
__device__ __forceinline__ void tr_row_edges(const TrArgs& A, int64_t i, int64_t n_src, F f) {
    int64_t b = A.row_start[i], e = A.row_end[i];
    if (b < 0) b = 0;
    if (e > A.max_nnz) e = A.max_nnz;
    for (int64_t k = b; k < e; ++k) {
        const int32_t c = A.col[k];
        if (c >= 0 && c < n_src) f((int32_t)i, c);
    }
}

__global__ __launch_bounds__(TR_THREADS) void transpose_count_kernel(TrArgs A) {
    const int64_t n = tr_count(A.n_dev, A.max_rows), n_src = tr_count(A.n_src_dev, A.max_src);
    const int64_t i = (int64_t)blockIdx.x * TR_THREADS + threadIdx.x;
    if (i < n) tr_row_edges(A, i, n_src, [&](int32_t, int32_t c) { atomicAdd(&A.cnt[c], 1); });
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void transpose_sum_kernel(TrArgs A) {
    __shared__ long long red[16];
    const int64_t j = (int64_t)blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    const long long s = fg_block_sum(j < A.max_src ? (long long)A.cnt[j] : 0, red);
    if (threadIdx.x == 0) A.blk[blockIdx.x] = (int32_t)s;
}

__global__ __launch_bounds__(FG_SCAN_BLOCK) void transpose_scan_kernel(TrArgs A) {
    __shared__ long long red[16];
    __shared__ int wave_sum[FG_SCAN_BLOCK / FG_WAVE];
    const int64_t j = (int64_t)blockIdx.x * FG_SCAN_BLOCK + threadIdx.x;
    long long before = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += FG_SCAN_BLOCK) before += A.blk[b];
    before = fg_block_sum(before, red);
    const int c = j < A.max_src ? A.cnt[j] : 0;
    int incl = c;  // inclusive scan over the wavefront, then the wavefronts before this one
    for (int off = 1; off < FG_WAVE; off <<= 1) {
        const int v = __shfl_up(incl, off, FG_WAVE);
        if (fg_lane() >= off) incl += v;
    }
    if (fg_lane() == FG_WAVE - 1) wave_sum[fg_wave()] = incl;
    __syncthreads();
    int earlier = 0;
    for (int w = 0; w < fg_wave(); ++w) earlier += wave_sum[w];
    if (j < A.max_src) {
        const long long first = before + earlier + incl - c;
        A.t_start[j] = (int32_t)first;
        A.t_end[j] = (int32_t)(first + c);
        A.cnt[j] = 0;  // from here on: the next free place of the list
    }
}

__global__ __launch_bounds__(TR_THREADS) void transpose_fill_kernel(TrArgs A) {
    const int64_t n = tr_count(A.n_dev, A.max_rows), n_src = tr_count(A.n_src_dev, A.max_src);
    const int64_t i = (int64_t)blockIdx.x * TR_THREADS + threadIdx.x;
    if (i < n)
        tr_row_edges(A, i, n_src, [&](int32_t row, int32_t c) {
            const int64_t at = (int64_t)A.t_start[c] + atomicAdd(&A.cnt[c], 1);
            if (at < A.max_nnz) A.t_row[at] = row;
        });
}

__global__ __launch_bounds__(TR_THREADS) void transpose_sort_kernel(TrArgs A) {
    const int64_t j = (int64_t)blockIdx.x * TR_THREADS + threadIdx.x;
    if (j >= A.max_src) return;
    int64_t b = A.t_start[j], e = A.t_end[j];
    if (e > A.max_nnz) e = A.max_nnz;
    for (int64_t k = b + 1; k < e; ++k) {  // insertion sort
        const int32_t v = A.t_row[k];
        int64_t q = k;
        while (q > b && A.t_row[q - 1] > v) {
            A.t_row[q] = A.t_row[q - 1];
            --q;
        }
        A.t_row[q] = v;
    }
}

size_t tr_layout(int64_t max_src, size_t* blk_at) {
    const size_t src = (size_t)(max_src > 0 ? max_src : 1);
    *blk_at = fg_align_up(src * 4, 256);
    return *blk_at + fg_align_up((size_t)fg_ceil_div((int64_t)src, FG_SCAN_BLOCK) * 4, 256);
}

}  // namespace

extern "C" size_t fg_transpose_block_workspace_bytes(int64_t max_src) {
    if (max_src < 0 || max_src > INT32_MAX) return 0;
    size_t at;
    return tr_layout(max_src, &at);
}

extern "C" fg_status_t fg_transpose_block(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                                          const int64_t* n_dev, int64_t max_rows, const int64_t* n_src_dev, int64_t max_src,
                                          int64_t max_nnz, int32_t* t_start_dev, int32_t* t_end_dev, int32_t* t_row_dev,
                                          void* ws_dev, size_t ws_bytes, void* stream) {
    const char* who = "fg_transpose_block";
    if (max_rows < 0 || max_src < 0 || max_nnz < 0 || max_rows > INT32_MAX || max_src > INT32_MAX || max_nnz > INT32_MAX)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: bad size (max_rows %lld, max_src %lld, max_nnz %lld)", who, (long long)max_rows,
                (long long)max_src, (long long)max_nnz);
    if (max_rows > 0 && (!row_start_dev || !row_end_dev || (max_nnz > 0 && !col_dev))) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL block", who);
    if (max_src > 0 && (!t_start_dev || !t_end_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL output", who);
    if (max_nnz > 0 && !t_row_dev) FG_FAIL(FG_ERR_INVALID_ARG, "%s: t_row_dev is NULL", who);
    size_t blk_at;
    const size_t need = tr_layout(max_src, &blk_at);
    if (max_src > 0 && (!ws_dev || ws_bytes < need)) FG_FAIL(FG_ERR_SHAPE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes, need);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: workspace must be 16-byte aligned", who);
    fg_clear_error();
    if (max_src == 0) return FG_OK;
    hipStream_t st = (hipStream_t)stream;
    TrArgs A{row_start_dev, row_end_dev, col_dev, n_dev, max_rows, n_src_dev, max_src, max_nnz, t_start_dev, t_end_dev, t_row_dev,
             (int32_t*)ws_dev, (int32_t*)((char*)ws_dev + blk_at)};
    fg_status_t rc = fg_launch_fill_i32(A.cnt, max_src, 0, st);
    if (rc != FG_OK) return rc;
    const unsigned row_blocks = (unsigned)fg_ceil_div(max_rows > 0 ? max_rows : 1, TR_THREADS);
    const unsigned scan_blocks = (unsigned)fg_ceil_div(max_src, FG_SCAN_BLOCK);
    if (max_rows > 0) {
        hipLaunchKernelGGL(transpose_count_kernel, dim3(row_blocks), dim3(TR_THREADS), 0, st, A);
        FG_LAUNCH_CHECK("transpose_count_kernel");
    }
    hipLaunchKernelGGL(transpose_sum_kernel, dim3(scan_blocks), dim3(FG_SCAN_BLOCK), 0, st, A);
    FG_LAUNCH_CHECK("transpose_sum_kernel");
    hipLaunchKernelGGL(transpose_scan_kernel, dim3(scan_blocks), dim3(FG_SCAN_BLOCK), 0, st, A);
    FG_LAUNCH_CHECK("transpose_scan_kernel");
    if (max_rows > 0) {
        hipLaunchKernelGGL(transpose_fill_kernel, dim3(row_blocks), dim3(TR_THREADS), 0, st, A);
        FG_LAUNCH_CHECK("transpose_fill_kernel");
        hipLaunchKernelGGL(transpose_sort_kernel, dim3((unsigned)fg_ceil_div(max_src, TR_THREADS)), dim3(TR_THREADS), 0, st, A);
        FG_LAUNCH_CHECK("transpose_sort_kernel");
    }
    return FG_OK;
}
