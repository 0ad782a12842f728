// fg_gather: dst[dst_pos[k], :] = table[src_index[k], :], a bit copy of whole rows.
//
// This is the loader of Algorithm 1 (Load_feature of the unpruned input nodes; Section 6: the device reads
// rows by node id straight from where the table lives, HBM or host memory mapped into its address space)
// and the fetch of cached embeddings C^(l)[v].
//
// HBM-bound: every byte is read once and written once. A row is split into 16-byte pieces over a group of
// 2^g lanes (a 512-byte row is one dwordx4 load per lane of half a wavefront), each group keeps UNROLL rows
// in flight, and a fixed-size grid walks the list so that the element count can stay in device memory.
#include "common.h"

namespace {

template <typename V, bool NT>
__device__ __forceinline__ V load_row_piece(const V* p) {
    if constexpr (NT)
        return __builtin_nontemporal_load(p);  // table rows are read once: do not displace what the next stages reuse
    else
        return *p;
}

// FEAT: src_index holds node ids, and a node whose row is still on the feature side of the shared buffer (Section 4.2)
// is read from there instead of from the table.
template <typename V, int UNROLL, bool NT, bool FEAT>
__global__ __launch_bounds__(256) void gather_rows_kernel(const char* __restrict__ table, int64_t table_rows,
                                                          int64_t src_stride, int chunks,
                                                          const int32_t* __restrict__ src_index,
                                                          const int32_t* __restrict__ dst_pos,
                                                          const int64_t* __restrict__ count_dev, int64_t max_count,
                                                          char* __restrict__ dst, int64_t dst_rows, int64_t dst_stride,
                                                          int lanes_log2, fg_feat_side F) {
    int64_t count = count_dev ? *count_dev : max_count;
    if (count > max_count) count = max_count;
    const int lanes = 1 << lanes_log2;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t group = gtid >> lanes_log2;
    const int lane = (int)(gtid & (lanes - 1));
    const int64_t ngroups = ((int64_t)gridDim.x * blockDim.x) >> lanes_log2;
    for (int64_t k0 = group; k0 < count; k0 += ngroups * UNROLL) {
        const V* src[UNROLL];
        V* out[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t k = k0 + (int64_t)u * ngroups;
            src[u] = nullptr;
            out[u] = nullptr;
            if (k < count) {
                const int64_t s = src_index[k];
                const int64_t d = dst_pos ? (int64_t)dst_pos[k] : k;
                if (s >= 0 && s < table_rows && d >= 0 && d < dst_rows) {
                    src[u] = (const V*)(table + s * src_stride);
                    if constexpr (FEAT) {
                        const int32_t r = fg_feature_rank(F, (int32_t)s);
                        if (r >= 0) src[u] = (const V*)(F.end - (int64_t)(r + 1) * F.row_bytes);
                    }
                    out[u] = (V*)(dst + d * dst_stride);
                }
            }
        }
        if (chunks <= lanes) {
            V v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (src[u] && lane < chunks) v[u] = load_row_piece<V, NT>(src[u] + lane);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (src[u] && lane < chunks) out[u][lane] = v[u];
        } else {
            for (int c = lane; c < chunks; c += lanes) {
                V v[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
                    if (src[u]) v[u] = load_row_piece<V, NT>(src[u] + c);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
                    if (src[u]) out[u][c] = v[u];
            }
        }
    }
}

// blockIdx.y selects the copy; a wavefront moves a row in 16-byte pieces, two rows in flight.
constexpr int COPY_THREADS = 256;
__global__ __launch_bounds__(COPY_THREADS) void copy_rows_batch_kernel(fg_row_copy_batch B) {
    fg_copy_rows_part(B.c[blockIdx.y], ((int64_t)blockIdx.x * COPY_THREADS + threadIdx.x) >> 6, ((int64_t)gridDim.x * COPY_THREADS) >> 6,
                      threadIdx.x & 63);
}

template <typename T>
__global__ void fill_kernel(T* p, int64_t n, T value) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = value;
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <typename V, int UNROLL, bool NT, bool FEAT>
void launch_gather_u(const void* table, int64_t table_rows, int64_t src_stride, int64_t row_bytes,
                     const int32_t* src_index, const int32_t* dst_pos, const int64_t* count_dev, int64_t max_count,
                     void* dst, int64_t dst_rows, int64_t dst_stride, int on_host, hipStream_t st, const fg_feat_side& F) {
    const int chunks = (int)(row_bytes / (int64_t)sizeof(V));
    int lg = 0;
    while ((1 << lg) < chunks && lg < 6) ++lg;
    const int lanes = 1 << lg;
    const int groups_per_block = 256 / lanes;
    int64_t blocks = fg_ceil_div(max_count, (int64_t)groups_per_block * UNROLL);
    // a few workgroups per compute unit; the grid loops over the list
    const int64_t cap = 256 * fg_tuning(on_host == 1 ? FG_TUNE_GATHER_HOST_WG_PER_CU : FG_TUNE_GATHER_WG_PER_CU);
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((gather_rows_kernel<V, UNROLL, NT, FEAT>), dim3((unsigned)blocks), dim3(256), 0, st, (const char*)table,
                       table_rows, src_stride, chunks, src_index, dst_pos, count_dev, max_count, (char*)dst, dst_rows,
                       dst_stride, lg, F);
}

template <typename V, bool FEAT = false>
void launch_gather_t(const void* table, int64_t table_rows, int64_t src_stride, int64_t row_bytes,
                     const int32_t* src_index, const int32_t* dst_pos, const int64_t* count_dev, int64_t max_count,
                     void* dst, int64_t dst_rows, int64_t dst_stride, int on_host, hipStream_t st,
                     const fg_feat_side& F = fg_feat_side{}) {
    const int unroll = (int)fg_tuning(FG_TUNE_GATHER_UNROLL);
    // rows of a big table are read once (streaming loads); rows that were just written or will be read again
    // (cached embeddings, layer outputs) go through the caches normally
    const bool nt = on_host != 2 && fg_tuning(FG_TUNE_GATHER_NONTEMPORAL) != 0;
#define FG_G(U, N)                                                                                                      \
    launch_gather_u<V, U, N, FEAT>(table, table_rows, src_stride, row_bytes, src_index, dst_pos, count_dev, max_count, \
                                   dst, dst_rows, dst_stride, on_host, st, F)
    if (unroll <= 1) { if (nt) FG_G(1, true); else FG_G(1, false); }
    else if (unroll == 2) { if (nt) FG_G(2, true); else FG_G(2, false); }
    else if (unroll <= 4) { if (nt) FG_G(4, true); else FG_G(4, false); }
    else { if (nt) FG_G(8, true); else FG_G(8, false); }
#undef FG_G
}

}  // namespace

fg_status_t fg_launch_row_copies(const fg_row_copy_batch& batch, hipStream_t stream) {
    int64_t most = 0;
    for (int i = 0; i < batch.n; ++i)
        if (batch.c[i].max_count > most) most = batch.c[i].max_count;
    if (batch.n <= 0 || most <= 0) return FG_OK;
    int64_t gx = fg_ceil_div(most, 2 * (COPY_THREADS / 64));
    if (gx > 2048) gx = 2048;
    hipLaunchKernelGGL(copy_rows_batch_kernel, dim3((unsigned)gx, (unsigned)batch.n), dim3(COPY_THREADS), 0, stream, batch);
    FG_LAUNCH_CHECK("copy_rows_batch_kernel");
    return FG_OK;
}

fg_status_t fg_launch_fill_u8(uint8_t* p, int64_t n, uint8_t value, hipStream_t stream) {
    if (n <= 0) return FG_OK;
    if ((((uintptr_t)p) & 3) == 0 && (n & 3) == 0) {
        const uint32_t v4 = 0x01010101u * value;
        const int64_t n4 = n / 4;
        const int blocks = (int)(fg_ceil_div(n4, 256) < 2048 ? fg_ceil_div(n4, 256) : 2048);
        hipLaunchKernelGGL(fill_kernel<uint32_t>, dim3(blocks), dim3(256), 0, stream, (uint32_t*)p, n4, v4);
    } else {
        const int blocks = (int)(fg_ceil_div(n, 256) < 2048 ? fg_ceil_div(n, 256) : 2048);
        hipLaunchKernelGGL(fill_kernel<uint8_t>, dim3(blocks), dim3(256), 0, stream, p, n, value);
    }
    FG_LAUNCH_CHECK("fill_kernel");
    return FG_OK;
}

fg_status_t fg_launch_fill_i32(int32_t* p, int64_t n, int32_t value, hipStream_t stream) {
    if (n <= 0) return FG_OK;
    const int blocks = (int)(fg_ceil_div(n, 256) < 4096 ? fg_ceil_div(n, 256) : 4096);
    hipLaunchKernelGGL(fill_kernel<int32_t>, dim3(blocks), dim3(256), 0, stream, p, n, value);
    FG_LAUNCH_CHECK("fill_kernel");
    return FG_OK;
}

fg_status_t fg_launch_gather(const void* table, int64_t table_rows, int64_t src_stride, int64_t row_bytes,
                             const int32_t* src_index, const int32_t* dst_pos, const int64_t* count_dev,
                             int64_t max_count, void* dst, int64_t dst_rows, int64_t dst_stride, int on_host,
                             hipStream_t st, const fg_feat_side* feat) {
    if (max_count == 0 || row_bytes == 0) return FG_OK;
    const uintptr_t bits = (uintptr_t)table | (uintptr_t)dst | (uintptr_t)src_stride | (uintptr_t)dst_stride | (uintptr_t)row_bytes;
    if (feat && feat->rank) {
        if (bits & 15) FG_FAIL(FG_ERR_INVALID_ARG, "gather through the feature side needs 16-byte aligned rows");
        launch_gather_t<u32x4, true>(table, table_rows, src_stride, row_bytes, src_index, dst_pos, count_dev, max_count, dst,
                                     dst_rows, dst_stride, on_host, st, *feat);
    } else if ((bits & 15) == 0)
        launch_gather_t<u32x4>(table, table_rows, src_stride, row_bytes, src_index, dst_pos, count_dev, max_count, dst,
                               dst_rows, dst_stride, on_host, st);
    else if ((bits & 7) == 0)
        launch_gather_t<u32x2>(table, table_rows, src_stride, row_bytes, src_index, dst_pos, count_dev, max_count, dst,
                               dst_rows, dst_stride, on_host, st);
    else if ((bits & 3) == 0)
        launch_gather_t<uint32_t>(table, table_rows, src_stride, row_bytes, src_index, dst_pos, count_dev, max_count,
                                  dst, dst_rows, dst_stride, on_host, st);
    else
        launch_gather_t<uint16_t>(table, table_rows, src_stride, row_bytes, src_index, dst_pos, count_dev, max_count,
                                  dst, dst_rows, dst_stride, on_host, st);
    FG_LAUNCH_CHECK("gather_rows_kernel");
    return FG_OK;
}

static fg_status_t gather_checked(const char* who, const fg_feat_side* feat, const void* table, int64_t table_rows,
                                  int64_t src_stride, int64_t row_bytes, const int32_t* src_index_dev,
                                  const int32_t* dst_pos_dev, const int64_t* count_dev, int64_t max_count, void* dst,
                                  int64_t dst_rows, int64_t dst_stride, int32_t table_kind, void* stream) {
    if (max_count < 0 || table_rows < 0 || dst_rows < 0 || row_bytes < 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: negative size (max_count %lld, table_rows %lld, dst_rows %lld, row_bytes %lld)", who,
                (long long)max_count, (long long)table_rows, (long long)dst_rows, (long long)row_bytes);
    if (max_count > 0 && row_bytes > 0 && (!table || !dst || !src_index_dev))
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: table, dst and src_index_dev are required", who);
    if (row_bytes & 1) FG_FAIL(FG_ERR_SHAPE, "%s: row_bytes = %lld is odd", who, (long long)row_bytes);
    if (src_stride < row_bytes || dst_stride < row_bytes)
        FG_FAIL(FG_ERR_SHAPE, "%s: a row stride (%lld, %lld) is smaller than row_bytes = %lld", who, (long long)src_stride,
                (long long)dst_stride, (long long)row_bytes);
    const uintptr_t bits = (uintptr_t)table | (uintptr_t)dst | (uintptr_t)src_stride | (uintptr_t)dst_stride;
    int64_t need = 16;
    while (need > 2 && (row_bytes % need) != 0) need >>= 1;
    if (bits & (uintptr_t)(need - 1))
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: pointers and strides must be %lld-byte aligned for rows of %lld bytes", who,
                (long long)need, (long long)row_bytes);
    if (table_kind < 0 || table_kind > 2) FG_FAIL(FG_ERR_INVALID_ARG, "%s: table_kind = %d is not FG_TABLE_*", who, table_kind);
    if (feat && feat->rank && max_count > 0 && row_bytes > 0) {
        if (row_bytes != feat->row_bytes)
            FG_FAIL(FG_ERR_SHAPE, "%s: row_bytes = %lld differs from the %lld-byte rows on the feature side", who, (long long)row_bytes,
                    (long long)feat->row_bytes);
        if (row_bytes % 16 || (bits & 15)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: rows, pointers and strides must be 16-byte aligned", who);
    }
    fg_clear_error();
    return fg_launch_gather(table, table_rows, src_stride, row_bytes, src_index_dev, dst_pos_dev, count_dev, max_count,
                            dst, dst_rows, dst_stride, table_kind, (hipStream_t)stream, feat);
}

extern "C" fg_status_t fg_gather(const void* table, int64_t table_rows, int64_t src_stride, int64_t row_bytes,
                                 const int32_t* src_index_dev, const int32_t* dst_pos_dev, const int64_t* count_dev,
                                 int64_t max_count, void* dst, int64_t dst_rows, int64_t dst_stride,
                                 int32_t table_kind, void* stream) {
    return gather_checked("fg_gather", nullptr, table, table_rows, src_stride, row_bytes, src_index_dev, dst_pos_dev, count_dev,
                          max_count, dst, dst_rows, dst_stride, table_kind, stream);
}

extern "C" fg_status_t fg_gather_features(const fg_cache_t* cache, const void* table, int64_t table_rows, int64_t src_stride,
                                          int64_t row_bytes, const int32_t* ids_dev, const int32_t* dst_pos_dev,
                                          const int64_t* count_dev, int64_t max_count, void* dst, int64_t dst_rows,
                                          int64_t dst_stride, int32_t table_kind, void* stream) {
    if (!cache) FG_FAIL(FG_ERR_INVALID_ARG, "fg_gather_features: cache is NULL");
    if (table_rows > cache->num_nodes)
        FG_FAIL(FG_ERR_SHAPE, "fg_gather_features: the table has %lld rows but the cache was created for %lld nodes", (long long)table_rows,
                (long long)cache->num_nodes);
    const fg_feat_side F = fg_feature_side(cache);
    return gather_checked("fg_gather_features", &F, table, table_rows, src_stride, row_bytes, ids_dev, dst_pos_dev, count_dev,
                          max_count, dst, dst_rows, dst_stride, table_kind, stream);
}
