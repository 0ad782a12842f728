// fg_aggregate: mean of the sampled neighbours' previous-layer rows (AGG of Eq. 1, mean aggregator) for the
// rows of V_normal, over the pruned two-row-array block.
//
// HBM/L2-bound: nnz rows of d elements are read, one row of d per output written. A group of 2^g lanes owns
// one output row and holds 16 bytes of it per lane (4 fp32 or 8 16-bit elements); the neighbour indices of
// the rows a workgroup works on are staged in LDS by a coalesced load and then read back as broadcasts,
// and the neighbour rows are fetched UNROLL at a time. Sums are carried in fp64 (the arithmetic is free
// next to the memory traffic) and rounded once, so the result does not depend on the neighbour order
// beyond fp64 rounding.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "common.h"

namespace {

constexpr int AGG_THREADS = 256;
constexpr int AGG_MAX_STAGE = 64;  // neighbour indices staged per row and pass
constexpr int AGG_UNROLL = 5;      // neighbour rows in flight per lane

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
struct Elem;
template <>
struct Elem<FG_F32> {
    static constexpr int PER16 = 4;
    __device__ static void unpack(const u32x4& raw, double* acc) {
        acc[0] += (double)__uint_as_float(raw.x);
        acc[1] += (double)__uint_as_float(raw.y);
        acc[2] += (double)__uint_as_float(raw.z);
        acc[3] += (double)__uint_as_float(raw.w);
    }
};
template <>
struct Elem<FG_F16> {
    static constexpr int PER16 = 8;
    __device__ static void unpack(const u32x4& raw, double* acc) {
        const unsigned int w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += (double)__half2float(__ushort_as_half((unsigned short)(w[i] & 0xFFFF)));
            acc[2 * i + 1] += (double)__half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
        }
    }
};
template <>
struct Elem<FG_BF16> {
    static constexpr int PER16 = 8;
    __device__ static void unpack(const u32x4& raw, double* acc) {
        const unsigned int w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += (double)__uint_as_float(w[i] << 16);
            acc[2 * i + 1] += (double)__uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};

// round an fp32 value to bf16 bits, nearest even (finite inputs)
__device__ __forceinline__ unsigned int bf16_bits(float f) {
    const unsigned int b = __float_as_uint(f);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ unsigned int half_bits(float f) { return (unsigned int)__half_as_ushort(__float2half_rn(f)); }

// acc / deg rounded once to OUT and written as aligned vector stores (N = 4 or 8 elements)
template <int OUT, int N>
__device__ __forceinline__ void store_row_piece(char* dst, const double* acc, double deg) {
    float v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = deg > 0.0 ? (float)(acc[i] / deg) : 0.0f;
    if constexpr (OUT == FG_F32) {
#pragma unroll
        for (int i = 0; i < N; i += 4) {
            f32x4 o = {v[i], v[i + 1], v[i + 2], v[i + 3]};
            *(f32x4*)(dst + 4 * i) = o;
        }
    } else {
        unsigned int w[N / 2];
#pragma unroll
        for (int i = 0; i < N / 2; ++i) {
            if constexpr (OUT == FG_BF16)
                w[i] = bf16_bits(v[2 * i]) | (bf16_bits(v[2 * i + 1]) << 16);
            else
                w[i] = half_bits(v[2 * i]) | (half_bits(v[2 * i + 1]) << 16);
        }
        if constexpr (N == 4) {
            u32x2 o = {w[0], w[1]};
            *(u32x2*)dst = o;
        } else {
            u32x4 o = {w[0], w[1], w[2], w[3]};
            *(u32x4*)dst = o;
        }
    }
}

// what a load reads where there is no neighbour row to read (its value is never used)
__device__ __attribute__((aligned(16))) unsigned int agg_spare[4];

template <bool STREAM>
__device__ __forceinline__ u32x4 load_piece(const char* p) {
    if constexpr (STREAM)
        return __builtin_nontemporal_load((const u32x4*)p);
    else
        return *(const u32x4*)p;
}

// IN: element type of h_src; OUT: element type of agg. One group of `lanes` lanes per output row;
// pieces = 16-byte pieces per row (may exceed `lanes`, then a lane loops).
// INDIRECT: h_src is a table indexed by node id and src_ids[] maps a neighbour position to its id (the fused
// loader + first-layer aggregation); table rows are then read with streaming loads, once each.
// FEAT (with INDIRECT): a node whose raw features are still on the feature side of the shared buffer (Section 4.2)
// is read from there. The staged entry of such a neighbour is -2 - rank instead of the node id.
// GCN: the propagation of a GCN layer in row-normalised form: the row's own previous embedding is part of the mean,
// (h_r + sum of the neighbours) / (deg + 1). The result is written as the two halves the dense update reads: columns
// [0, dim/2) to gcn_pos[r, :] (by position), columns [dim/2, dim) to agg[k, :] (list order).
// COLIDS (with INDIRECT): col[] already holds table rows (node ids), so the position -> id step is skipped for the
// neighbours; src_ids is then only used for the rows' own ids.
template <int IN, int OUT, bool INDIRECT, bool FEAT, bool GCN = false, bool COLIDS = false>
__device__ __forceinline__ void aggregate_mean_body(
    const int n_blocks, const int block,  // workgroups doing this work and this workgroup's number among them
    const int32_t* __restrict__ row_start, const int32_t* __restrict__ row_end, const int32_t* __restrict__ col,
    int64_t nnz, int n_block_rows, const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev,
    int64_t max_rows, const char* __restrict__ h_src, int64_t n_src, int64_t src_stride, int pieces, char* __restrict__ agg,
    int64_t agg_stride, int lanes_log2, const int32_t* __restrict__ src_ids, int n_ids, char* __restrict__ self_out,
    int64_t self_stride, int n_self, fg_feat_side F, char* __restrict__ gcn_pos, int64_t gcn_pos_stride) {
    constexpr int PER = Elem<IN>::PER16;
    constexpr int OUT_BYTES = (OUT == FG_F32 ? 4 : 2) * PER;
    extern __shared__ int32_t nb_lds[];  // [groups_per_block][AGG_MAX_STAGE]
    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    const int lanes = 1 << lanes_log2;
    const int gpb = AGG_THREADS >> lanes_log2;
    const int g_in_block = threadIdx.x >> lanes_log2;
    const int lane = threadIdx.x & (lanes - 1);
    int32_t* my_nb = nb_lds + g_in_block * AGG_MAX_STAGE;
    for (int64_t k = (int64_t)block * gpb + g_in_block; k < n_rows; k += (int64_t)n_blocks * gpb) {
        const int32_t r = rows ? rows[k] : (int32_t)k;
        int32_t s0 = 0, e0 = 0;
        if (r >= 0 && r < n_block_rows) {
            s0 = row_start[r];
            e0 = row_end[r];
            if (s0 < 0 || e0 < s0 || (int64_t)e0 > nnz) e0 = s0 = 0;
        }
        const int deg = e0 - s0;
        // fused loader: the row's own features (position r of the input layer is the same node) go to self_out[r]
        const char* self_row = nullptr;
        if (GCN && !INDIRECT && r >= 0 && r < n_src && r < n_block_rows) self_row = h_src + (int64_t)r * src_stride;
        if (INDIRECT && (self_out || GCN) && r >= 0 && r < n_ids && (GCN ? r < n_block_rows : r < n_self)) {
            const int32_t v = src_ids[r];
            if (v >= 0 && v < n_src) {
                self_row = h_src + (int64_t)v * src_stride;
                if constexpr (FEAT) {
                    const int32_t fr = fg_feature_rank(F, v);
                    if (fr >= 0) self_row = F.end - (int64_t)(fr + 1) * F.row_bytes;
                }
            }
        }
        for (int p0 = 0; p0 < pieces; p0 += lanes) {
            const int piece = p0 + lane;
            const bool active = piece < pieces;
            u32x4 self_piece;
            if ((INDIRECT || GCN) && self_row && active) self_piece = load_piece<INDIRECT>(self_row + (int64_t)piece * 16);
            double acc[PER];
#pragma unroll
            for (int i = 0; i < PER; ++i) acc[i] = 0.0;
            if (GCN && self_row && active) Elem<IN>::unpack(self_piece, acc);
            const int deg_ld = n_src > 0 ? deg : 0;  // an empty source has no row to read (the means are then zero)
            for (int base = 0; base < deg_ld; base += AGG_MAX_STAGE) {
                const int cnt = min(deg_ld - base, AGG_MAX_STAGE);
                // stage this row's neighbour positions: coalesced read, broadcast reads afterwards
                for (int t = lane; t < cnt; t += lanes) {
                    int32_t c = col[s0 + base + t];
                    if (INDIRECT && !COLIDS) c = (c >= 0 && c < n_ids) ? src_ids[c] : -1;
                    if constexpr (FEAT) {
                        if (c >= 0 && c < n_src) {
                            const int32_t fr = fg_feature_rank(F, c);
                            if (fr >= 0) c = -2 - fr;
                        }
                    }
                    my_nb[t] = c;
                }
                // lanes of a group sit in one wavefront when lanes <= 64, so LDS writes above are visible
                // to the group after a wavefront-level fence
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                // AGG_UNROLL neighbour rows in flight per lane, issued back to back without branches: a slot past the
                // end of the row (or an out-of-range index) reads 16 bytes of the library's own (agg_spare, the same
                // for every lane: a cache hit) and is dropped when the values are added up. Re-reading a row of the
                // batch instead costs a second trip to memory: with streaming loads that row is not in a cache while
                // its first read is still in flight (the loader: 78 -> 73 us). Nothing touches a loaded value before
                // the whole batch has been issued.
                if constexpr (FEAT) {
                    // the same batching with a row address per neighbour: the table, or the feature side for an entry <= -2
                    auto row_of = [&](int32_t c) -> const char* {
                        if (c <= -2) return F.end - (int64_t)(-1 - c) * F.row_bytes;  // rank -2-c starts at end - (rank+1)*row
                        return (c >= 0 && c < n_src) ? h_src + (int64_t)c * src_stride : nullptr;
                    };
                    for (int t = 0; t < cnt; t += AGG_UNROLL) {
                        u32x4 raw[AGG_UNROLL];
                        bool ok[AGG_UNROLL];
#pragma unroll
                        for (int u = 0; u < AGG_UNROLL; ++u) {
                            const char* p = (t + u < cnt) ? row_of(my_nb[t + u]) : nullptr;
                            ok[u] = p != nullptr;
                            raw[u] = load_piece<INDIRECT>(ok[u] ? p + (int64_t)(active ? piece : 0) * 16 : (const char*)agg_spare);
                        }
#pragma unroll
                        for (int u = 0; u < AGG_UNROLL; ++u)
                            if (ok[u]) Elem<IN>::unpack(raw[u], acc);
                    }
                } else
                for (int t = 0; t < cnt; t += AGG_UNROLL) {
                    u32x4 raw[AGG_UNROLL];
                    bool ok[AGG_UNROLL];
#pragma unroll
                    for (int u = 0; u < AGG_UNROLL; ++u) {
                        const int32_t c = (t + u < cnt) ? my_nb[t + u] : -1;
                        ok[u] = c >= 0 && c < n_src;
                        raw[u] = load_piece<INDIRECT>(ok[u] ? h_src + (int64_t)c * src_stride + (int64_t)(active ? piece : 0) * 16
                                                            : (const char*)agg_spare);
                    }
#pragma unroll
                    for (int u = 0; u < AGG_UNROLL; ++u)
                        if (ok[u]) Elem<IN>::unpack(raw[u], acc);
                }
                __builtin_amdgcn_wave_barrier();  // the stage is rewritten by the next pass
            }
            if constexpr (GCN) {
                const int half = pieces >> 1;
                if (active && self_row) {
                    char* dst = piece < half ? gcn_pos + (int64_t)r * gcn_pos_stride + (int64_t)piece * OUT_BYTES
                                             : agg + k * agg_stride + (int64_t)(piece - half) * OUT_BYTES;
                    store_row_piece<OUT, PER>(dst, acc, (double)(deg + 1));
                }
            } else {
                if (active) store_row_piece<OUT, PER>(agg + k * agg_stride + (int64_t)piece * OUT_BYTES, acc, (double)deg);
            }
            if constexpr (GCN) {
                if (INDIRECT && self_out && self_row && r < n_self && active)
                    *(u32x4*)(self_out + (int64_t)r * self_stride + (int64_t)piece * 16) = self_piece;
            } else {
                if (INDIRECT && self_row && active) *(u32x4*)(self_out + (int64_t)r * self_stride + (int64_t)piece * 16) = self_piece;
            }
        }
    }
}


template <int IN, int OUT, bool INDIRECT, bool FEAT, bool GCN = false, bool COLIDS = false>
__global__ __launch_bounds__(AGG_THREADS) void aggregate_mean_kernel(
    const int32_t* __restrict__ row_start, const int32_t* __restrict__ row_end, const int32_t* __restrict__ col,
    int64_t nnz, int n_block_rows, const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev,
    int64_t max_rows, const char* __restrict__ h_src, int64_t n_src, int64_t src_stride, int pieces, char* __restrict__ agg,
    int64_t agg_stride, int lanes_log2, const int32_t* __restrict__ src_ids, int n_ids, char* __restrict__ self_out,
    int64_t self_stride, int n_self, fg_feat_side F, char* __restrict__ gcn_pos = nullptr, int64_t gcn_pos_stride = 0) {
    aggregate_mean_body<IN, OUT, INDIRECT, FEAT, GCN, COLIDS>(gridDim.x, blockIdx.x, row_start, row_end, col, nnz, n_block_rows, rows,
                                                              n_rows_dev, max_rows, h_src, n_src, src_stride, pieces, agg, agg_stride,
                                                              lanes_log2, src_ids, n_ids, self_out, self_stride, n_self, F, gcn_pos,
                                                              gcn_pos_stride);
}

// The fused loader with the fetch of cached embeddings riding along: the first copy_blocks workgroups copy the cached rows
// of the hits of every cached layer (h_v = C^(l)[v] of Algorithm 1), the remaining ones are the loader. The two jobs do
// not depend on each other; sharing a launch saves one of the path's small launches. The copies come first in the grid:
// the loader's workgroups stay resident until the end of the launch, so workgroups behind them would only start then
// (with a few thousand hits per mini-batch that was a tail of tens of microseconds).
template <int IN, int OUT>
__global__ __launch_bounds__(AGG_THREADS) void loader_fetch_kernel(
    int copy_blocks, fg_row_copy_batch copies, const int32_t* __restrict__ row_start, const int32_t* __restrict__ row_end,
    const int32_t* __restrict__ col, int64_t nnz, int n_block_rows, const int32_t* __restrict__ rows,
    const int64_t* __restrict__ n_rows_dev, int64_t max_rows, const char* __restrict__ h_src, int64_t n_src, int64_t src_stride,
    int pieces, char* __restrict__ agg, int64_t agg_stride, int lanes_log2, const int32_t* __restrict__ src_ids, int n_ids,
    char* __restrict__ self_out, int64_t self_stride, int n_self) {
    if ((int)blockIdx.x < copy_blocks) {
        const int64_t wave = ((int64_t)blockIdx.x * AGG_THREADS + threadIdx.x) >> 6;
        const int64_t n_waves = ((int64_t)copy_blocks * AGG_THREADS) >> 6;
        for (int c = 0; c < copies.n; ++c) fg_copy_rows_part(copies.c[c], wave, n_waves, threadIdx.x & 63);
        return;
    }
    aggregate_mean_body<IN, OUT, true, false, false, true>((int)gridDim.x - copy_blocks, (int)blockIdx.x - copy_blocks, row_start, row_end, col, nnz, n_block_rows, rows,
                                                          n_rows_dev, max_rows, h_src, n_src, src_stride, pieces, agg, agg_stride,
                                                          lanes_log2, src_ids, n_ids, self_out, self_stride, n_self, fg_feat_side{},
                                                          nullptr, 0);
}

}  // namespace

// Lanes (as a power of two) that share one row of `pieces` 16-byte pieces.  A row wider than a
// wavefront is walked in passes; when the last pass of 64 lanes would sit half idle (96 pieces: a
// 1536-byte row) groups of 32 lanes, two rows per wavefront, leave none idle and the loader over
// host-resident features runs 8 % faster.  Rows of whole multiples of 64 pieces keep 64 lanes.
static int lanes_log2_for(int pieces) {
    int lg = 0;
    while ((1 << lg) < pieces && lg < 6) ++lg;
    if (lg == 6 && (pieces + 31) / 32 * 32 < (pieces + 63) / 64 * 64) lg = 5;
    return lg;
}

static fg_status_t aggregate_common(const char* who, const int32_t* row_start_dev, const int32_t* row_end_dev,
                                    const int32_t* col_dev, int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev,
                                    const int64_t* n_rows_dev, int64_t max_rows, const void* h_src, int64_t n_src,
                                    int64_t src_stride, int32_t dim, fg_dtype_t in_dtype, void* agg, int64_t agg_stride,
                                    fg_dtype_t out_dtype, const int32_t* src_ids, int32_t n_ids, void* self_out,
                                    int64_t self_stride, int32_t n_self, void* stream, const fg_feat_side* feat = nullptr,
                                    void* gcn_pos = nullptr, int64_t gcn_pos_stride = 0, bool col_is_ids = false) {
    if (max_rows < 0 || n_block_rows < 0 || n_src < 0 || dim <= 0 || nnz < 0 || n_ids < 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: bad size (max_rows %lld, n_block_rows %d, n_src %lld, dim %d, nnz %lld)", who,
                (long long)max_rows, n_block_rows, (long long)n_src, dim, (long long)nnz);
    const int isz = fg_dtype_size(in_dtype), osz = fg_dtype_size(out_dtype);
    if (!isz || !osz) FG_FAIL(FG_ERR_DTYPE, "%s: unknown element type", who);
    if (max_rows > 0 && (!row_start_dev || !row_end_dev || !h_src || !agg || (nnz > 0 && !col_dev)))
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    const int per16 = 16 / isz;
    if (dim % per16) FG_FAIL(FG_ERR_SHAPE, "%s: dim = %d must be a multiple of %d for this type", who, dim, per16);
    if (src_stride < (int64_t)dim * isz || agg_stride < (int64_t)dim * osz / (gcn_pos ? 2 : 1))
        FG_FAIL(FG_ERR_SHAPE, "%s: row stride smaller than a row", who);
    if (((uintptr_t)h_src | (uintptr_t)src_stride) & 15)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: the source rows and their stride must be 16-byte aligned", who);
    if (((uintptr_t)agg | (uintptr_t)agg_stride) & 15)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: agg and its stride must be 16-byte aligned", who);
    fg_clear_error();
    if (max_rows == 0) return FG_OK;
    const int pieces = dim / per16;
    const int lg = lanes_log2_for(pieces);
    const int gpb = AGG_THREADS >> lg;
    int64_t blocks = fg_ceil_div(max_rows, gpb);
    const int64_t cap = 256 * fg_tuning(FG_TUNE_AGG_WG_PER_CU);
    if (blocks > cap) blocks = cap;
    const size_t lds = (size_t)gpb * AGG_MAX_STAGE * sizeof(int32_t);
    hipStream_t st = (hipStream_t)stream;
    const bool with_feat = feat && feat->rank && src_ids;
    if (with_feat && feat->row_bytes != (int64_t)dim * isz)
        FG_FAIL(FG_ERR_SHAPE, "%s: rows of %lld bytes differ from the %lld-byte rows on the feature side", who, (long long)dim * isz,
                (long long)feat->row_bytes);
    const fg_feat_side F = with_feat ? *feat : fg_feat_side{};
    if (gcn_pos) {  // GCN propagation: fp32, halves of the mean to gcn_pos (by position) and agg (list order)
        if (src_ids)
            hipLaunchKernelGGL((aggregate_mean_kernel<FG_F32, FG_F32, true, false, true>), dim3((unsigned)blocks), dim3(AGG_THREADS), lds,
                               st, row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows,
                               (const char*)h_src, n_src, src_stride, pieces, (char*)agg, agg_stride, lg, src_ids, n_ids,
                               (char*)self_out, self_stride, n_self, F, (char*)gcn_pos, gcn_pos_stride);
        else
            hipLaunchKernelGGL((aggregate_mean_kernel<FG_F32, FG_F32, false, false, true>), dim3((unsigned)blocks), dim3(AGG_THREADS), lds,
                               st, row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows,
                               (const char*)h_src, n_src, src_stride, pieces, (char*)agg, agg_stride, lg, src_ids, n_ids,
                               (char*)self_out, self_stride, n_self, F, (char*)gcn_pos, gcn_pos_stride);
        FG_LAUNCH_CHECK("aggregate_mean_kernel (GCN)");
        return FG_OK;
    }
#define FG_AGG_LAUNCH_F(IN, OUT, IND, FT)                                                                              \
    hipLaunchKernelGGL((aggregate_mean_kernel<IN, OUT, IND, FT>), dim3((unsigned)blocks), dim3(AGG_THREADS), lds, st,   \
                       row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows,          \
                       (const char*)h_src, n_src, src_stride, pieces, (char*)agg, agg_stride, lg, src_ids, n_ids,       \
                       (char*)self_out, self_stride, n_self, F)
#define FG_AGG_LAUNCH(IN, OUT, IND)                       \
    do {                                                  \
        if constexpr (IND) {                              \
            if (with_feat)                                \
                FG_AGG_LAUNCH_F(IN, OUT, true, true);     \
            else if (col_is_ids)                          \
                hipLaunchKernelGGL((aggregate_mean_kernel<IN, OUT, true, false, false, true>), dim3((unsigned)blocks),       \
                                   dim3(AGG_THREADS), lds, st, row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, \
                                   n_rows_dev, max_rows, (const char*)h_src, n_src, src_stride, pieces, (char*)agg, agg_stride,  \
                                   lg, src_ids, n_ids, (char*)self_out, self_stride, n_self, F);                                 \
            else                                          \
                FG_AGG_LAUNCH_F(IN, OUT, true, false);    \
        } else {                                          \
            FG_AGG_LAUNCH_F(IN, OUT, false, false);       \
        }                                                 \
    } while (0)
#define FG_AGG_OUT(IN, IND)                            \
    do {                                               \
        if (out_dtype == FG_F32)                       \
            FG_AGG_LAUNCH(IN, FG_F32, IND);            \
        else if (out_dtype == FG_F16)                  \
            FG_AGG_LAUNCH(IN, FG_F16, IND);            \
        else                                           \
            FG_AGG_LAUNCH(IN, FG_BF16, IND);           \
    } while (0)
#define FG_AGG_IN(IND)                                 \
    do {                                               \
        if (in_dtype == FG_F32)                        \
            FG_AGG_OUT(FG_F32, IND);                   \
        else if (in_dtype == FG_F16)                   \
            FG_AGG_OUT(FG_F16, IND);                   \
        else                                           \
            FG_AGG_OUT(FG_BF16, IND);                  \
    } while (0)
    if (src_ids)
        FG_AGG_IN(true);
    else
        FG_AGG_IN(false);
#undef FG_AGG_IN
#undef FG_AGG_OUT
#undef FG_AGG_LAUNCH
#undef FG_AGG_LAUNCH_F
    FG_LAUNCH_CHECK("aggregate_mean_kernel");
    return FG_OK;
}

extern "C" fg_status_t fg_aggregate(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                                    int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev,
                                    const int64_t* n_rows_dev, int64_t max_rows, const void* h_src, int32_t n_src,
                                    int64_t src_stride, int32_t dim, fg_dtype_t in_dtype, void* agg, int64_t agg_stride,
                                    fg_dtype_t out_dtype, void* stream) {
    return aggregate_common("fg_aggregate", row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev,
                            max_rows, h_src, n_src, src_stride, dim, in_dtype, agg, agg_stride, out_dtype, nullptr, 0, nullptr, 0,
                            0, stream);
}

static fg_status_t gather_aggregate_checked(const char* who, const fg_feat_side* feat, const int32_t* row_start_dev,
                                            const int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz,
                                            int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                            int64_t max_rows, const int32_t* src_ids_dev, int32_t n_src, const void* table,
                                            int64_t table_rows, int64_t src_stride, int32_t dim, fg_dtype_t in_dtype, void* agg,
                                            int64_t agg_stride, fg_dtype_t out_dtype, void* h_self_out, int64_t h_self_stride,
                                            int32_t n_self_rows, void* stream) {
    if (max_rows > 0 && !src_ids_dev) FG_FAIL(FG_ERR_INVALID_ARG, "%s: src_ids_dev is NULL", who);
    if (h_self_out) {
        if (n_self_rows < 0 || h_self_stride < (int64_t)dim * fg_dtype_size(in_dtype))
            FG_FAIL(FG_ERR_SHAPE, "%s: h_self_out needs n_self_rows >= 0 and a stride of at least one row", who);
        if (((uintptr_t)h_self_out | (uintptr_t)h_self_stride) & 15)
            FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_self_out and its stride must be 16-byte aligned", who);
    }
    return aggregate_common(who, row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows, table,
                            table_rows, src_stride, dim, in_dtype, agg, agg_stride, out_dtype, src_ids_dev, n_src, h_self_out,
                            h_self_stride, n_self_rows, stream, feat);
}

extern "C" fg_status_t fg_gather_aggregate(const int32_t* row_start_dev, const int32_t* row_end_dev,
                                           const int32_t* col_dev, int64_t nnz, int32_t n_block_rows,
                                           const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                                           const int32_t* src_ids_dev, int32_t n_src, const void* table, int64_t table_rows,
                                           int64_t src_stride, int32_t dim, fg_dtype_t in_dtype, void* agg,
                                           int64_t agg_stride, fg_dtype_t out_dtype, void* h_self_out,
                                           int64_t h_self_stride, int32_t n_self_rows, void* stream) {
    return gather_aggregate_checked("fg_gather_aggregate", nullptr, row_start_dev, row_end_dev, col_dev, nnz, n_block_rows,
                                    rows_dev, n_rows_dev, max_rows, src_ids_dev, n_src, table, table_rows, src_stride, dim,
                                    in_dtype, agg, agg_stride, out_dtype, h_self_out, h_self_stride, n_self_rows, stream);
}

extern "C" fg_status_t fg_gather_aggregate_ids(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_ids_dev,
                                               int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                               int64_t max_rows, const int32_t* row_ids_dev, const void* table, int64_t table_rows,
                                               int64_t src_stride, int32_t dim, fg_dtype_t in_dtype, void* agg, int64_t agg_stride,
                                               fg_dtype_t out_dtype, void* h_self_out, int64_t h_self_stride, int32_t n_self_rows,
                                               const fg_cache_t* cache, int32_t n_fetch_layers, const fg_fetch_layer_t* fetch_layers,
                                               void* stream) {
    const char* who = "fg_gather_aggregate_ids";
    if (max_rows > 0 && !row_ids_dev) FG_FAIL(FG_ERR_INVALID_ARG, "%s: row_ids_dev is NULL", who);
    if (h_self_out) {
        if (n_self_rows < 0 || h_self_stride < (int64_t)dim * fg_dtype_size(in_dtype))
            FG_FAIL(FG_ERR_SHAPE, "%s: h_self_out needs n_self_rows >= 0 and a stride of at least one row", who);
        if (((uintptr_t)h_self_out | (uintptr_t)h_self_stride) & 15)
            FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_self_out and its stride must be 16-byte aligned", who);
    }
    fg_row_copy_batch copies;
    copies.n = 0;
    if (n_fetch_layers != 0) {
        fg_status_t rc = fg_build_fetch_batch(who, cache, n_fetch_layers, fetch_layers, &copies);
        if (rc != FG_OK) return rc;
    }
    int64_t most = 0;
    for (int i = 0; i < copies.n; ++i) most = copies.c[i].max_count > most ? copies.c[i].max_count : most;
    const bool f32 = in_dtype == FG_F32 && out_dtype == FG_F32, h16 = in_dtype == FG_F16 && out_dtype == FG_BF16;
    if (most == 0 || max_rows <= 0 || !(f32 || h16)) {  // nothing to fetch, or a type pair without the shared launch: two launches
        if (most > 0) {
            fg_status_t rc = fg_launch_row_copies(copies, (hipStream_t)stream);
            if (rc != FG_OK) return rc;
        }
        return aggregate_common(who, row_start_dev, row_end_dev, col_ids_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows, table,
                                table_rows, src_stride, dim, in_dtype, agg, agg_stride, out_dtype, row_ids_dev, n_block_rows,
                                h_self_out, h_self_stride, n_self_rows, stream, nullptr, nullptr, 0, true);
    }
    // the loader's own checks, without launching it
    fg_status_t rc = aggregate_common(who, row_start_dev, row_end_dev, col_ids_dev, nnz, n_block_rows, rows_dev, n_rows_dev, 0, table,
                                      table_rows, src_stride, dim, in_dtype, agg, agg_stride, out_dtype, row_ids_dev, n_block_rows,
                                      h_self_out, h_self_stride, n_self_rows, stream, nullptr, nullptr, 0, true);
    if (rc != FG_OK) return rc;
    if (!row_start_dev || !row_end_dev || !table || !agg || (nnz > 0 && !col_ids_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    const int per16 = 16 / fg_dtype_size(in_dtype);
    const int pieces = dim / per16;
    const int lg = lanes_log2_for(pieces);
    const int gpb = AGG_THREADS >> lg;
    int64_t blocks = fg_ceil_div(max_rows, gpb);
    const int64_t cap = 256 * fg_tuning(FG_TUNE_AGG_WG_PER_CU);
    if (blocks > cap) blocks = cap;
    // sized by the bound on the hits (their number is known on the device only): a wavefront copies two rows at a time
    int64_t copy_blocks = fg_ceil_div(most, 8 * (AGG_THREADS / 64));
    if (copy_blocks > 256) copy_blocks = 256;
    const size_t lds = (size_t)gpb * AGG_MAX_STAGE * sizeof(int32_t);
    hipStream_t st = (hipStream_t)stream;
    if (f32)
        hipLaunchKernelGGL((loader_fetch_kernel<FG_F32, FG_F32>), dim3((unsigned)(blocks + copy_blocks)), dim3(AGG_THREADS), lds, st,
                           (int)copy_blocks, copies, row_start_dev, row_end_dev, col_ids_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows,
                           (const char*)table, table_rows, src_stride, pieces, (char*)agg, agg_stride, lg, row_ids_dev, n_block_rows,
                           (char*)h_self_out, h_self_stride, n_self_rows);
    else
        hipLaunchKernelGGL((loader_fetch_kernel<FG_F16, FG_BF16>), dim3((unsigned)(blocks + copy_blocks)), dim3(AGG_THREADS), lds, st,
                           (int)copy_blocks, copies, row_start_dev, row_end_dev, col_ids_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows,
                           (const char*)table, table_rows, src_stride, pieces, (char*)agg, agg_stride, lg, row_ids_dev, n_block_rows,
                           (char*)h_self_out, h_self_stride, n_self_rows);
    FG_LAUNCH_CHECK("loader_fetch_kernel");
    return FG_OK;
}

extern "C" fg_status_t fg_gather_aggregate_features(const fg_cache_t* cache, const int32_t* row_start_dev,
                                                    const int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz,
                                                    int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                                    int64_t max_rows, const int32_t* src_ids_dev, int32_t n_src,
                                                    const void* table, int64_t table_rows, int64_t src_stride, int32_t dim,
                                                    fg_dtype_t in_dtype, void* agg, int64_t agg_stride, fg_dtype_t out_dtype,
                                                    void* h_self_out, int64_t h_self_stride, int32_t n_self_rows,
                                                    void* stream) {
    if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "fg_gather_aggregate_features: cache is NULL");
    if (table_rows > cache->num_nodes)
        FG_FAIL(FG_ERR_SHAPE, "fg_gather_aggregate_features: the table has %lld rows but the cache was created for %lld nodes",
                (long long)table_rows, (long long)cache->num_nodes);
    const fg_feat_side F = fg_feature_side(cache);
    return gather_aggregate_checked("fg_gather_aggregate_features", &F, row_start_dev, row_end_dev, col_dev, nnz, n_block_rows,
                                    rows_dev, n_rows_dev, max_rows, src_ids_dev, n_src, table, table_rows, src_stride, dim,
                                    in_dtype, agg, agg_stride, out_dtype, h_self_out, h_self_stride, n_self_rows, stream);
}


// GCN propagation (row-normalised graph convolution with the node itself included), fp32:
//   m[k, :] = (h_src[r, :] + sum_{e in [row_start[r], row_end[r])} h_src[col[e], :]) / (deg + 1),  r = rows[k]
// written as the two K-halves fg_linear reads: m[k, 0:dim/2] -> mean_pos[r, :], m[k, dim/2:dim] -> mean_cmp[k, :].
static fg_status_t aggregate_gcn_checked(const char* who, const int32_t* row_start_dev, const int32_t* row_end_dev,
                                         const int32_t* col_dev, int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev,
                                         const int64_t* n_rows_dev, int64_t max_rows, const int32_t* src_ids_dev, int32_t n_ids,
                                         const void* h_src, int64_t n_src, int64_t src_stride, int32_t dim, void* mean_pos,
                                         void* mean_cmp, void* h_self_out, int64_t h_self_stride, int32_t n_self_rows, void* stream) {
    if (dim <= 0 || dim % 8) FG_FAIL(FG_ERR_SHAPE, "%s: dim = %d must be a positive multiple of 8", who, dim);
    if (max_rows > 0 && (!mean_pos || !mean_cmp)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: mean_pos_dev and mean_cmp_dev are required", who);
    if (((uintptr_t)mean_pos | (uintptr_t)mean_cmp) & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: the outputs must be 16-byte aligned", who);
    const int64_t half_bytes = (int64_t)dim / 2 * 4;
    return aggregate_common(who, row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows, h_src, n_src,
                            src_stride, dim, FG_F32, mean_cmp, half_bytes, FG_F32, src_ids_dev, n_ids, h_self_out, h_self_stride,
                            n_self_rows, stream, nullptr, mean_pos, half_bytes);
}

extern "C" fg_status_t fg_aggregate_gcn(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz,
                                        int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                                        const float* h_src, int32_t n_src, int64_t src_stride, int32_t dim, float* mean_pos_dev,
                                        float* mean_cmp_dev, void* stream) {
    return aggregate_gcn_checked("fg_aggregate_gcn", row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows,
                                 nullptr, 0, h_src, n_src, src_stride, dim, mean_pos_dev, mean_cmp_dev, nullptr, 0, 0, stream);
}

extern "C" fg_status_t fg_gather_aggregate_gcn(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                                               int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                               int64_t max_rows, const int32_t* src_ids_dev, int32_t n_src, const float* table,
                                               int64_t table_rows, int64_t src_stride, int32_t dim, float* mean_pos_dev,
                                               float* mean_cmp_dev, void* stream) {
    if (max_rows > 0 && !src_ids_dev) FG_FAIL(FG_ERR_INVALID_ARG, "fg_gather_aggregate_gcn: src_ids_dev is NULL");
    return aggregate_gcn_checked("fg_gather_aggregate_gcn", row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev,
                                 max_rows, src_ids_dev, n_src, table, table_rows, src_stride, dim, mean_pos_dev, mean_cmp_dev, nullptr, 0,
                                 0, stream);
}
