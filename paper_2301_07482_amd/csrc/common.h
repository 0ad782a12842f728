// Internal declarations shared by the translation units of libfreshgnn (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "freshgnn.h"

struct fg_layer {
    int64_t capacity = 0;
    int32_t dim = 0;
    int32_t* map = nullptr;         // [num_nodes] slot of each node or -1
    int32_t* slot_node = nullptr;   // [capacity] owner of each slot or -1
    int32_t* slot_stamp = nullptr;  // [capacity] iteration whose update filled the slot
    void* table = nullptr;          // [capacity x dim], inside the cache's shared buffer at byte offset `base`
    int64_t base = 0;
    int64_t* head = nullptr;        // device int64[4]: ring header, double-buffered (head_cur indexes the current one);
                                    // [2] = slots written at least once (0 .. used-1: the ring fills upwards until it wraps)
    int head_cur = 0;
    void* sel = nullptr;            // selection scratch of the update (two histograms and a count), all-zero between updates
    int64_t last_iter = INT64_MIN;  // host: iteration of the last update
    bool copy_pending = false;      // host: fg_cache_update_select has run for last_iter, fg_cache_update_commit not yet
};

struct fg_cache {
    int64_t num_nodes = 0;
    int32_t n_layers = 0;
    fg_dtype_t dtype = FG_F32;
    int32_t t_stale = 0;
    int64_t stabilization = 0;   // iterations before this one neither look the cache up nor admit into it (Section 4.1.4)
    fg_layer* layers = nullptr;  // host array [n_layers], layer l at index l-1
    // the buffer embeddings and raw features share (Section 4.2): rings from the left end in layer order,
    // feature rows from the right end, rank r at [buffer_bytes - (r+1)*feat_row_bytes, buffer_bytes - r*feat_row_bytes)
    char* buffer = nullptr;
    int64_t buffer_bytes = 0;
    int32_t* feat_rank = nullptr;  // [num_nodes] rank of a node's row on the feature side or -1; allocated by the first fill
    int64_t n_feat = 0;            // feature rows placed (0: no feature side)
    int64_t feat_row_bytes = 0;
};

constexpr int FG_MAX_RINGS = 8;       // cached layers a feature side can share its buffer with
constexpr int64_t FG_RING_ALIGN = 256;  // a ring's first byte in the shared buffer is a multiple of this

// What a kernel needs to find a node's raw feature row on the feature side of the shared buffer.
struct fg_feat_side {
    const int32_t* rank;  // nullptr: nothing placed
    const char* end;      // one past the buffer: the row of rank r starts at end - (r+1)*row_bytes
    int64_t row_bytes, n_rows, buffer_bytes;
    int32_t n_rings;
    int64_t ring_lo[FG_MAX_RINGS];           // first byte of each ring
    int64_t ring_row[FG_MAX_RINGS];          // bytes per slot
    const int64_t* ring_used[FG_MAX_RINGS];  // device: slots written so far
};
fg_feat_side fg_feature_side(const fg_cache_t* cache);

// Rank of node v's row (0 <= v < num_nodes) if it was placed and no embedding has been written over any of its
// bytes, else -1. A ring has written exactly the bytes of its slots 0 .. used-1.
__device__ __forceinline__ int32_t fg_feature_rank(const fg_feat_side& F, int32_t v) {
    int32_t r = F.rank[v];
    if (r < 0 || r >= F.n_rows) return -1;
    const int64_t lo = F.buffer_bytes - (int64_t)(r + 1) * F.row_bytes, hi = lo + F.row_bytes;
#pragma unroll
    for (int i = 0; i < FG_MAX_RINGS; ++i) {
        if (i < F.n_rings) {
            const int64_t used = *F.ring_used[i];
            const int64_t w_lo = F.ring_lo[i], w_hi = w_lo + used * F.ring_row[i];
            if (used > 0 && lo < w_hi && hi > w_lo) r = -1;
        }
    }
    return r;
}

// staleness bound in force for a lookup at iteration `iter`: none is usable during the stabilization period
static inline int32_t fg_t_stale_at(const fg_cache_t* c, int64_t iter) { return iter < c->stabilization ? 0 : c->t_stale; }

void fg_set_error(const char* fmt, ...);
void fg_clear_error();

static inline int fg_dtype_size(fg_dtype_t t) { return t == FG_F32 ? 4 : (t == FG_F16 || t == FG_BF16) ? 2 : 0; }

#define FG_FAIL(code, ...)         \
    do {                           \
        fg_set_error(__VA_ARGS__); \
        return (code);             \
    } while (0)

#define FG_HIP(expr)                                                                       \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess) FG_FAIL(FG_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// Returns FG_ERR_HIP if the launch just queued was rejected.
#define FG_LAUNCH_CHECK(name)                                                                          \
    do {                                                                                               \
        hipError_t e_ = hipGetLastError();                                                             \
        if (e_ != hipSuccess) FG_FAIL(FG_ERR_HIP, "launch of %s failed: %s", name, hipGetErrorString(e_)); \
    } while (0)

constexpr int FG_SCAN_BLOCK = 1024;  // elements (= threads) per block in the compaction kernels

static inline int64_t fg_ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t fg_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// launch-shape parameters (defaults tuned on MI355X; fg_set_tuning overrides them for measurements)
enum fg_tune_id {
    FG_TUNE_GATHER_WG_PER_CU = 0,
    FG_TUNE_GATHER_HOST_WG_PER_CU,
    FG_TUNE_GATHER_UNROLL,
    FG_TUNE_GATHER_NONTEMPORAL,
    FG_TUNE_AGG_WG_PER_CU,
    FG_TUNE_LINEAR_TILE,  // 0: choose by problem size; 8: split-K kernel, 32: panel kernel, 64 or 128: LDS-tiled kernel; bf16: 1064, 1128
    FG_TUNE_TOP_DOWN_WALK,  // 1: fg_top_down walks the first two blocks from the seeds in its first launch; 0: one layer per launch
    FG_TUNE_COUNT
};
int64_t fg_tuning(fg_tune_id id);

// internal row copy used by fg_gather and by the cache update; feat (may be NULL, else 16-byte rows) makes
// src_index node ids whose rows are taken from the feature side where they are still there
fg_status_t fg_launch_gather(const void* table, int64_t table_rows, int64_t src_stride, int64_t row_bytes,
                             const int32_t* src_index, const int32_t* dst_pos, const int64_t* count_dev,
                             int64_t max_count, void* dst, int64_t dst_rows, int64_t dst_stride, int on_host,
                             hipStream_t stream, const fg_feat_side* feat = nullptr);
// Several independent row copies in one launch: dst[dst_idx[k], :] = src[src_idx[k], :] for k < *count (rows a
// multiple of 16 bytes, 16-byte aligned). Used where a pass copies rows for every cached layer at once.
constexpr int FG_MAX_COPIES = 8;
struct fg_row_copy {
    const char* src;
    int64_t src_rows, src_stride;
    const int32_t* src_idx;
    const int32_t* dst_idx;
    const int64_t* count;  // device
    int64_t max_count;
    char* dst;
    int64_t dst_rows, dst_stride;
    int64_t row_bytes;
};
struct fg_row_copy_batch {
    int32_t n;
    fg_row_copy c[FG_MAX_COPIES];
};
fg_status_t fg_launch_row_copies(const fg_row_copy_batch& batch, hipStream_t stream);
// the copy work of wavefront `wave` of `n_waves`: a wavefront moves a row in 16-byte pieces, two rows in flight
__device__ __forceinline__ void fg_copy_rows_part(const fg_row_copy& C, int64_t wave, int64_t n_waves, int lane) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    int64_t count = C.count ? *C.count : C.max_count;
    if (count > C.max_count) count = C.max_count;
    const int chunks = (int)(C.row_bytes >> 4);
    for (int64_t k0 = wave; k0 < count; k0 += 2 * n_waves) {
        const int64_t k1 = k0 + n_waves;
        const bool has1 = k1 < count;
        const int32_t s0 = C.src_idx[k0], d0 = C.dst_idx ? C.dst_idx[k0] : (int32_t)k0;
        const int32_t s1 = has1 ? C.src_idx[k1] : s0, d1 = has1 ? (C.dst_idx ? C.dst_idx[k1] : (int32_t)k1) : d0;
        const bool ok0 = s0 >= 0 && s0 < C.src_rows && d0 >= 0 && d0 < C.dst_rows;
        const bool ok1 = has1 && s1 >= 0 && s1 < C.src_rows && d1 >= 0 && d1 < C.dst_rows;
        const u32x4* a0 = (const u32x4*)(C.src + (int64_t)(ok0 ? s0 : 0) * C.src_stride);
        const u32x4* a1 = (const u32x4*)(C.src + (int64_t)(ok1 ? s1 : 0) * C.src_stride);
        u32x4* o0 = (u32x4*)(C.dst + (int64_t)(ok0 ? d0 : 0) * C.dst_stride);
        u32x4* o1 = (u32x4*)(C.dst + (int64_t)(ok1 ? d1 : 0) * C.dst_stride);
        for (int c = lane; c < chunks; c += 64) {
            const u32x4 v0 = a0[c];
            const u32x4 v1 = a1[c];
            if (ok0) o0[c] = v0;
            if (ok1) o1[c] = v1;
        }
    }
}
// checks the layers of a cache fetch (as fg_cache_fetch_all does) and describes them as row copies
fg_status_t fg_build_fetch_batch(const char* who, const fg_cache_t* cache, int32_t n_layers, const fg_fetch_layer_t* layers,
                                 fg_row_copy_batch* out);
// fill n bytes with a value (a kernel, so that callers may capture it into a graph)
fg_status_t fg_launch_fill_u8(uint8_t* p, int64_t n, uint8_t value, hipStream_t stream);
fg_status_t fg_launch_fill_i32(int32_t* p, int64_t n, int32_t value, hipStream_t stream);
