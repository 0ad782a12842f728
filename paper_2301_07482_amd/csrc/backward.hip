// Backward pass of the GraphSAGE-mean layers as far as the embedding gradients (Algorithm 1: loss, loss.backward();
// Section 4.1.1: the norms of dL/dh are what admission to and check-out from the historical cache are decided on).
//
//   fg_softmax_xent_grad   dL/dH(L) of the mean softmax cross-entropy over the seeds
//   fg_layer_backward      dL/dH(l-1) from dL/dH(l) for one layer: ReLU mask, [d_self ‖ d_agg] = dz . W^T on the
//                          matrix cores (the forward GEMM path with transposed weights), then the transposed mean
//                          aggregation as a gather over the block's transpose (no atomics: every output row has one
//                          writer and the sums are carried in fp64, so the result does not depend on scheduling)
//   fg_row_norms           L2 norm per row
//
// Only rows that were computed (V_normal) pass gradient down; a fetched row receives its gradient and stops there.
// All of it is small next to the forward pass: the layer below the lowest cached one needs no input gradient.
#include "common.h"
#include <hip/hip_fp16.h>

namespace {

constexpr int BW_THREADS = 256;
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double wave_sum(double v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ double wave_max(double v) {
    for (int off = 32; off > 0; off >>= 1) {
        const double o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// one wavefront per row: p = softmax(h[i, :]) in fp64, dh[i, c] = (p[c] - [c == label]) / n
__global__ __launch_bounds__(BW_THREADS) void softmax_xent_grad_kernel(const char* __restrict__ h, int64_t h_stride,
                                                                       const int32_t* __restrict__ labels, int n, int d,
                                                                       char* __restrict__ dh, int64_t dh_stride) {
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = ((int64_t)gridDim.x * BW_THREADS) >> 6;
    for (int64_t i = ((int64_t)blockIdx.x * BW_THREADS + threadIdx.x) >> 6; i < n; i += n_waves) {
        const float* row = (const float*)(h + i * h_stride);
        double m = -1.0e300;
        for (int c = lane; c < d; c += 64) {
            const double v = (double)row[c];
            m = v > m ? v : m;
        }
        m = wave_max(m);
        double s = 0.0;
        for (int c = lane; c < d; c += 64) s += exp((double)row[c] - m);
        s = wave_sum(s);
        const int32_t y = labels[i];
        float* out = (float*)(dh + i * dh_stride);
        for (int c = lane; c < d; c += 64) {
            const double p = exp((double)row[c] - m) / s;
            out[c] = (float)((p - (c == y ? 1.0 : 0.0)) / (double)n);
        }
    }
}

// one wavefront per row: sqrt of the fp64 sum of squares
__global__ __launch_bounds__(BW_THREADS) void row_norms_kernel(const char* __restrict__ x, int64_t stride, int n, int d,
                                                               float* __restrict__ norms) {
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = ((int64_t)gridDim.x * BW_THREADS) >> 6;
    for (int64_t i = ((int64_t)blockIdx.x * BW_THREADS + threadIdx.x) >> 6; i < n; i += n_waves) {
        const float* row = (const float*)(x + i * stride);
        double s = 0.0;
        for (int c = lane; c < d; c += 64) {
            const double v = (double)row[c];
            s += v * v;
        }
        s = wave_sum(s);
        if (lane == 0) norms[i] = (float)sqrt(s);
    }
}

// round an fp32 value to bf16 bits, nearest even (finite inputs)
__device__ __forceinline__ unsigned short bw_bf16_bits(float f) {
    const unsigned int b = __float_as_uint(f);
    return (unsigned short)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float bw_bf16_value(unsigned short b) { return __uint_as_float((unsigned int)b << 16); }

// dz = dh[r, :] * (h[r, :] > 0) for r = rows[k]. The GEMM that follows takes its first K/2 input columns from a
// matrix indexed by position and the other K/2 from one indexed by list order, so dz is written in that form:
// columns [0, half) to dz_pos[r, :], columns [half, d) to dz_cmp[k, :].
// BF16: the layer's output h is bf16 and dz is rounded to bf16 (the operand type of the bf16 matrix product that follows).
// one 32 x 32 tile of wt[c, a] = w[a, c]; w is [rows x cols]
template <typename T>
__device__ __forceinline__ void transpose_tile(const T* __restrict__ w, int rows, int cols, T* __restrict__ wt, int bx, int by) {
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int c0 = bx * 32, a0 = by * 32;
    for (int i = ty; i < 32; i += 8)
        if (a0 + i < rows && c0 + tx < cols) tile[i][tx] = w[(int64_t)(a0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && a0 + tx < rows) wt[(int64_t)(c0 + i) * rows + a0 + tx] = tile[tx][i];
}

// The first t_blocks workgroups (t_gx of them per row of tiles) transpose the layer's fp32 weights for the product that
// follows, an independent job that would otherwise be a launch of its own; the others mask the gradient.
template <bool BF16>
__global__ __launch_bounds__(BW_THREADS) void relu_backward_kernel(const char* __restrict__ dh, int64_t dh_stride,
                                                                   const char* __restrict__ h, int64_t h_stride, int n,
                                                                   const int32_t* __restrict__ rows,
                                                                   const int64_t* __restrict__ n_rows_dev, int64_t max_rows,
                                                                   int d, void* __restrict__ dz_pos_v, void* __restrict__ dz_cmp_v,
                                                                   int t_blocks, int t_gx, const float* __restrict__ w, int w_rows,
                                                                   int w_cols, float* __restrict__ wt) {
    if ((int)blockIdx.x < t_blocks) {      // uniform over the workgroup
        transpose_tile<float>(w, w_rows, w_cols, wt, (int)blockIdx.x % t_gx, (int)blockIdx.x / t_gx);
        return;
    }
    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    const int half = d >> 1;
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = ((int64_t)(gridDim.x - t_blocks) * BW_THREADS) >> 6;
    for (int64_t k = ((int64_t)(blockIdx.x - t_blocks) * BW_THREADS + threadIdx.x) >> 6; k < n_rows; k += n_waves) {
        const int32_t r = rows ? rows[k] : (int32_t)k;
        if (r < 0 || r >= n) continue;
        const float* g = (const float*)(dh + (int64_t)r * dh_stride);
        const char* a = h ? h + (int64_t)r * h_stride : nullptr;
        for (int c = lane; c < d; c += 64) {
            float v = g[c];
            if (a) {
                const float act = BF16 ? bw_bf16_value(((const unsigned short*)a)[c]) : ((const float*)a)[c];
                if (!(act > 0.f)) v = 0.f;
            }
            if constexpr (BF16) {
                const unsigned short b = bw_bf16_bits(v);
                if (c < half)
                    ((unsigned short*)dz_pos_v)[(int64_t)r * half + c] = b;
                else
                    ((unsigned short*)dz_cmp_v)[k * half + (c - half)] = b;
            } else {
                if (c < half)
                    ((float*)dz_pos_v)[(int64_t)r * half + c] = v;
                else
                    ((float*)dz_cmp_v)[k * half + (c - half)] = v;
            }
        }
    }
}

// Transposed mean aggregation. A group of 2^g lanes owns source position j and 16 bytes of the row per lane:
//   out[j, :] = [j is a computed row] dx[j, 0:d_in]  +  sum over t in [t_start[j], t_end[j]) with r = t_row[t] computed:
//               dx[r, d_in:2*d_in] / deg(r),   deg(r) = row_end[r] - row_start[r] of the pruned block
// A row that was not computed has an empty range in the pruned block (deg = 0) and is skipped by that test; such rows of
// dx were never written. Every position j < n_src is written (zeros where nothing arrives).
// GCN: the transpose of the propagation (h_r + sum of the neighbours) / (deg + 1): dx has d_in columns, and
//   out[j, :] = [j computed] dx[j, :] / (deg(j) + 1)  +  sum over the computed rows r that sampled j of dx[r, :] / (deg(r) + 1)
// (a row found in a transposed list sampled at least one neighbour, so it is computed exactly when deg(r) > 0).
// one source position j by a group of `lanes` lanes (this lane: `lane`); s0 .. e0 is its range of the transposed block
template <bool GCN>
__device__ __forceinline__ void aggregate_backward_row(
    const int64_t j, const int32_t s0, const int32_t e0, const int lane, const int lanes, const char* __restrict__ dx, int n, int d_in,
    const uint8_t* __restrict__ live, const uint8_t* __restrict__ hit, const int32_t* __restrict__ row_start,
    const int32_t* __restrict__ row_end, const int32_t* __restrict__ t_row, char* __restrict__ out, int64_t out_stride,
    float* __restrict__ norms) {
    const int pieces = d_in >> 2;
    const int64_t dx_stride = (int64_t)(GCN ? 1 : 2) * d_in * 4;
    const int nb_col = GCN ? 0 : d_in;      // first column of the neighbours' share in a row of dx
    const bool own = j < n && (live ? live[j] != 0 : true) && (hit ? hit[j] == 0 : true);
    double own_w = 1.0;
    if (GCN && own) {
        const int32_t deg = row_end[j] - row_start[j];
        own_w = 1.0 / (double)((deg > 0 ? deg : 0) + 1);
    }
    double ss = 0.0;  // this lane's share of the row's sum of squares (of the fp32 values written)
    for (int piece = lane; piece < pieces; piece += lanes) {
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        if (own) {
            const f32x4 v = *(const f32x4*)(dx + j * dx_stride + (int64_t)piece * 16);
            acc[0] = (double)v.x * own_w; acc[1] = (double)v.y * own_w; acc[2] = (double)v.z * own_w; acc[3] = (double)v.w * own_w;
        }
        for (int t = s0; t < e0; t += 4) {
            f32x4 v[4];
            double w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                w[u] = 0.0;
                v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (t + u < e0) {
                    const int32_t r = t_row[t + u];
                    if (r >= 0 && r < n) {
                        const int32_t deg = row_end[r] - row_start[r];
                        if (deg > 0) {
                            w[u] = 1.0 / (double)(GCN ? deg + 1 : deg);
                            v[u] = *(const f32x4*)(dx + (int64_t)r * dx_stride + (int64_t)(nb_col + 4 * piece) * 4);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc[0] += (double)v[u].x * w[u];
                acc[1] += (double)v[u].y * w[u];
                acc[2] += (double)v[u].z * w[u];
                acc[3] += (double)v[u].w * w[u];
            }
        }
        const f32x4 o = {(float)acc[0], (float)acc[1], (float)acc[2], (float)acc[3]};
        *(f32x4*)(out + j * out_stride + (int64_t)piece * 16) = o;
        ss += (double)o.x * o.x + (double)o.y * o.y + (double)o.z * o.z + (double)o.w * o.w;
    }
    if (norms) {  // the lanes of a group are neighbours in one wavefront and leave the loop together
        for (int off = lanes >> 1; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
        if (lane == 0) norms[j] = (float)sqrt(ss);
    }
}

// Groups of 2^lanes_log2 lanes take the source positions in turn. Where a group is smaller than a wavefront (several rows,
// several chains of index reads, per wavefront: what a layer with many rows wants), a position with more than `many`
// incoming edges is left out of that sweep and taken by a whole wavefront in a second one (by other workgroups of the same
// launch): a small group walks the edge list
// once per piece it holds, which for the hubs of a power-law graph was the whole launch (measured: 166 us against 84 us
// with one row per wavefront on the workload with average degree 50). Every position is written by exactly one group.
template <bool GCN>
__global__ __launch_bounds__(BW_THREADS) void aggregate_backward_kernel(
    const char* __restrict__ dx, int n, int d_in, const uint8_t* __restrict__ live, const uint8_t* __restrict__ hit,
    const int32_t* __restrict__ row_start, const int32_t* __restrict__ row_end, const int32_t* __restrict__ t_start,
    const int32_t* __restrict__ t_end, const int32_t* __restrict__ t_row, int64_t nnz, int n_src, char* __restrict__ out,
    int64_t out_stride, int lanes_log2, float* __restrict__ norms, int many, int sweep2_blocks) {
    const int lanes = 1 << lanes_log2;
    const int lane = threadIdx.x & (lanes - 1);
    const int gpb = BW_THREADS >> lanes_log2;
    const bool two_sweeps = lanes < 64;
    if ((int)blockIdx.x < sweep2_blocks) {
        // second sweep, by workgroups of its own at the front of the grid (the long rows start first): a wavefront looks
        // at 64 positions at once (one coalesced read of their ranges) and takes those with many incoming edges one after the
        // other, all 64 lanes on each
        const int wl = threadIdx.x & 63;
        const int64_t n_waves = (int64_t)sweep2_blocks * (BW_THREADS >> 6);
        for (int64_t j0 = ((int64_t)blockIdx.x * (BW_THREADS >> 6) + (threadIdx.x >> 6)) * 64; j0 < n_src; j0 += n_waves * 64) {
            int32_t s = 0, e = 0;
            if (j0 + wl < n_src) {
                s = t_start[j0 + wl];
                e = t_end[j0 + wl];
                if (s < 0 || e < s || (int64_t)e > nnz) s = e = 0;
            }
            unsigned long long big = __ballot(e - s > many);
            while (big) {      // uniform over the wavefront
                const int b = __ffsll((long long)big) - 1;
                big &= big - 1;
                const int32_t s0 = __shfl(s, b, 64), e0 = __shfl(e, b, 64);
                aggregate_backward_row<GCN>(j0 + b, s0, e0, wl, 64, dx, n, d_in, live, hit, row_start, row_end, t_row, out, out_stride, norms);
            }
        }
        return;
    }
    const int64_t block = (int64_t)blockIdx.x - sweep2_blocks, n_blocks = (int64_t)gridDim.x - sweep2_blocks;
    for (int64_t j = block * gpb + (threadIdx.x >> lanes_log2); j < n_src; j += n_blocks * gpb) {
        int32_t s0 = t_start[j], e0 = t_end[j];
        if (s0 < 0 || e0 < s0 || (int64_t)e0 > nnz) s0 = e0 = 0;
        if (two_sweeps && e0 - s0 > many) continue;
        aggregate_backward_row<GCN>(j, s0, e0, lane, lanes, dx, n, d_in, live, hit, row_start, row_end, t_row, out, out_stride, norms);
    }
}

struct BwWs {
    size_t dz_pos, dz_cmp, wt, dx, total;
};
// esz: bytes per element of dz and of the transposed weights (4, or 2 in the bf16 setting); cols: columns of dx
BwWs bw_layout(int64_t n, int64_t max_rows, int64_t cols, int64_t d_out, int64_t esz) {
    BwWs w;
    const size_t half = (size_t)(d_out / 2) * esz;
    w.dz_pos = 0;
    w.dz_cmp = fg_align_up((size_t)(n > 0 ? n : 1) * half, 256);
    w.wt = w.dz_cmp + fg_align_up((size_t)(max_rows > 0 ? max_rows : 1) * half, 256);
    w.dx = w.wt + fg_align_up((size_t)cols * d_out * esz, 256);
    w.total = w.dx + fg_align_up((size_t)(n > 0 ? n : 1) * cols * 4, 256);
    return w;
}

}  // namespace

fg_status_t fg_launch_linear_bf16(const void* h_src, int32_t n_src, int64_t src_stride, fg_dtype_t in_dtype, const void* agg,
                                  int64_t agg_stride, const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                                  int32_t d_in, int32_t d_out, const void* W, const float* bias, int32_t relu, void* h_out,
                                  int32_t n_out, int64_t out_stride, fg_dtype_t out_dtype, hipStream_t st, bool w_nk, const int64_t* k_limit_dev = nullptr,
                                  const int32_t* src_ids_dev = nullptr);

extern "C" fg_status_t fg_softmax_xent_grad(const float* h_dev, int64_t h_stride, const int32_t* labels_dev, int32_t n, int32_t d,
                                            float* dh_dev, int64_t dh_stride, void* stream) {
    if (n < 0 || d <= 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_softmax_xent_grad: bad size (n %d, d %d)", n, d);
    if (n > 0 && (!h_dev || !labels_dev || !dh_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "fg_softmax_xent_grad: NULL pointer");
    if (h_stride < (int64_t)d * 4 || dh_stride < (int64_t)d * 4) FG_FAIL(FG_ERR_SHAPE, "fg_softmax_xent_grad: a row stride is smaller than a row");
    if (((uintptr_t)h_dev | (uintptr_t)dh_dev | (uintptr_t)h_stride | (uintptr_t)dh_stride) & 3)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_softmax_xent_grad: pointers and strides must be 4-byte aligned");
    fg_clear_error();
    if (n == 0) return FG_OK;
    int64_t blocks = fg_ceil_div(n, BW_THREADS / 64);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(softmax_xent_grad_kernel, dim3((unsigned)blocks), dim3(BW_THREADS), 0, (hipStream_t)stream, (const char*)h_dev,
                       h_stride, labels_dev, n, d, (char*)dh_dev, dh_stride);
    FG_LAUNCH_CHECK("softmax_xent_grad_kernel");
    return FG_OK;
}

extern "C" fg_status_t fg_row_norms(const float* x_dev, int64_t x_stride, int32_t n, int32_t d, float* norms_dev, void* stream) {
    if (n < 0 || d <= 0) FG_FAIL(FG_ERR_INVALID_ARG, "fg_row_norms: bad size (n %d, d %d)", n, d);
    if (n > 0 && (!x_dev || !norms_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "fg_row_norms: NULL pointer");
    if (x_stride < (int64_t)d * 4) FG_FAIL(FG_ERR_SHAPE, "fg_row_norms: the row stride is smaller than a row");
    if (((uintptr_t)x_dev | (uintptr_t)x_stride | (uintptr_t)norms_dev) & 3) FG_FAIL(FG_ERR_INVALID_ARG, "fg_row_norms: pointers and stride must be 4-byte aligned");
    fg_clear_error();
    if (n == 0) return FG_OK;
    int64_t blocks = fg_ceil_div(n, BW_THREADS / 64);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(row_norms_kernel, dim3((unsigned)blocks), dim3(BW_THREADS), 0, (hipStream_t)stream, (const char*)x_dev, x_stride, n,
                       d, norms_dev);
    FG_LAUNCH_CHECK("row_norms_kernel");
    return FG_OK;
}

// kind of layer a backward call is for
enum BwKind { BW_SAGE_F32 = 0, BW_GCN_F32 = 1, BW_SAGE_BF16 = 2 };

static size_t layer_backward_ws(int kind, int32_t n, int64_t max_rows, int32_t d_in, int32_t d_out) {
    if (n < 0 || max_rows < 0 || d_in <= 0 || d_out <= 0) return 0;
    return bw_layout(n, max_rows, kind == BW_GCN_F32 ? d_in : 2 * (int64_t)d_in, d_out, kind == BW_SAGE_BF16 ? 2 : 4).total;
}

extern "C" size_t fg_layer_backward_workspace_bytes(int32_t n, int64_t max_rows, int32_t d_in, int32_t d_out) {
    return layer_backward_ws(BW_SAGE_F32, n, max_rows, d_in, d_out);
}
extern "C" size_t fg_layer_backward_gcn_workspace_bytes(int32_t n, int64_t max_rows, int32_t d_in, int32_t d_out) {
    return layer_backward_ws(BW_GCN_F32, n, max_rows, d_in, d_out);
}
extern "C" size_t fg_layer_backward_bf16_workspace_bytes(int32_t n, int64_t max_rows, int32_t d_in, int32_t d_out) {
    return layer_backward_ws(BW_SAGE_BF16, n, max_rows, d_in, d_out);
}

// The three layer kinds share the sequence: mask (+ rounding), transposed weights, dz . W^T on the forward GEMM path, transposed
// aggregation with the row norms.
static fg_status_t layer_backward_launch(const char* who, int kind, const float* dh_dev, int64_t dh_stride, const void* h_dev,
                                         int64_t h_stride, int32_t n, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                         int64_t max_rows, const uint8_t* live_dev, const uint8_t* hit_dev,
                                         const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* t_start_dev,
                                         const int32_t* t_end_dev, const int32_t* t_row_dev, int64_t nnz, int32_t n_src, int32_t d_in,
                                         int32_t d_out, const void* W, float* dh_src_dev, int64_t dh_src_stride, float* norms_src_dev,
                                         void* ws_dev, size_t ws_bytes, void* stream) {
    const bool gcn = kind == BW_GCN_F32, b16 = kind == BW_SAGE_BF16;
    const int esz = b16 ? 2 : 4;
    if (n < 0 || max_rows < 0 || n_src < 0 || nnz < 0 || d_in <= 0 || d_out <= 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: bad size (n %d, max_rows %lld, n_src %d, nnz %lld, d_in %d, d_out %d)", who, n, (long long)max_rows,
                n_src, (long long)nnz, d_in, d_out);
    if (n_src < n) FG_FAIL(FG_ERR_SHAPE, "%s: the layer below (%d positions) must contain this layer's %d", who, n_src, n);
    if (max_rows > n) FG_FAIL(FG_ERR_SHAPE, "%s: max_rows = %lld exceeds the layer's %d positions", who, (long long)max_rows, n);
    if (d_in % (b16 ? 8 : 4) || d_out % (b16 ? 16 : 8))
        FG_FAIL(FG_ERR_SHAPE, "%s: d_in = %d must be a multiple of %d and d_out = %d of %d", who, d_in, b16 ? 8 : 4, d_out, b16 ? 16 : 8);
    if (n_src > 0 && (!dh_src_dev || !t_start_dev || !t_end_dev || (nnz > 0 && !t_row_dev))) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (n > 0 && (!dh_dev || !row_start_dev || !row_end_dev || !W)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (dh_stride < (int64_t)d_out * 4 || (h_dev && h_stride < (int64_t)d_out * esz) || dh_src_stride < (int64_t)d_in * 4)
        FG_FAIL(FG_ERR_SHAPE, "%s: a row stride is smaller than its row", who);
    if (((uintptr_t)dh_dev | (uintptr_t)dh_stride) & 3 || ((uintptr_t)h_dev | (uintptr_t)h_stride) & (uintptr_t)(esz - 1))
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: dh, h and their strides must be aligned to their element size", who);
    if ((uintptr_t)W & (b16 ? 15 : 3)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: W must be %d-byte aligned", who, b16 ? 16 : 4);
    if ((uintptr_t)norms_src_dev & 3) FG_FAIL(FG_ERR_INVALID_ARG, "%s: norms_src_dev must be 4-byte aligned", who);
    if (((uintptr_t)dh_src_dev | (uintptr_t)dh_src_stride | (uintptr_t)ws_dev) & 15)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: dh_src_dev, its stride and the workspace must be 16-byte aligned", who);
    const int cols = gcn ? d_in : 2 * d_in;       // columns of dz . W^T
    const BwWs L = bw_layout(n, max_rows, cols, d_out, esz);
    if (!ws_dev || ws_bytes < L.total) FG_FAIL(FG_ERR_SHAPE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes, L.total);
    fg_clear_error();
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)ws_dev;
    void* dz_pos = ws + L.dz_pos;
    void* dz_cmp = ws + L.dz_cmp;
    void* wt = ws + L.wt;
    float* dx = (float*)(ws + L.dx);
    const int half = d_out / 2;
    if (n > 0 && max_rows > 0) {
        int64_t blocks = fg_ceil_div(max_rows, BW_THREADS / 64);
        if (blocks > 4096) blocks = 4096;
        const dim3 tgrid((unsigned)fg_ceil_div(d_out, 32), (unsigned)fg_ceil_div(cols, 32));
        if (b16) {
            hipLaunchKernelGGL(relu_backward_kernel<true>, dim3((unsigned)blocks), dim3(BW_THREADS), 0, st, (const char*)dh_dev, dh_stride,
                               (const char*)h_dev, h_stride, n, rows_dev, n_rows_dev, max_rows, d_out, dz_pos, dz_cmp, 0, 1,
                               (const float*)nullptr, 0, 0, (float*)nullptr);
            FG_LAUNCH_CHECK("relu_backward_kernel");
            // dx[r, :] = [dz_pos[r, :] ‖ dz_cmp[k, :]] . W^T, bf16 operands, fp32 sums and result. The weights of this product are
            // W^T; the matrix-core kernel takes them transposed, which is W as the caller holds it: nothing to transpose
            fg_status_t rc = fg_launch_linear_bf16(dz_pos, n, (int64_t)half * 2, FG_BF16, dz_cmp, (int64_t)half * 2, rows_dev, n_rows_dev,
                                                   max_rows, half, cols, W, nullptr, 0, dx, n, (int64_t)cols * 4, FG_F32, st, true);
            if (rc != FG_OK) return rc;
        } else {
            // (the transposition of W rides in the same launch: tgrid.x * tgrid.y workgroups in front of the others)
            const int t_blocks = (int)(tgrid.x * tgrid.y);
            hipLaunchKernelGGL(relu_backward_kernel<false>, dim3((unsigned)(blocks + t_blocks)), dim3(BW_THREADS), 0, st, (const char*)dh_dev,
                               dh_stride, (const char*)h_dev, h_stride, n, rows_dev, n_rows_dev, max_rows, d_out, dz_pos, dz_cmp, t_blocks,
                               (int)tgrid.x, (const float*)W, cols, d_out, (float*)wt);
            FG_LAUNCH_CHECK("relu_backward_kernel");
            // dx[r, :] = [dz_pos[r, :] ‖ dz_cmp[k, :]] . W^T for r = rows[k]: the forward GEMM with K = d_out, N = cols
            fg_status_t rc = fg_linear(dz_pos, n, (int64_t)half * 4, FG_F32, dz_cmp, (int64_t)half * 4, rows_dev, n_rows_dev, max_rows, half,
                                       cols, wt, FG_F32, nullptr, 0, dx, n, (int64_t)cols * 4, FG_F32, stream);
            if (rc != FG_OK) return rc;
        }
    }
    if (n_src == 0) return FG_OK;
    const int pieces = d_in / 4;
    // lanes per source row: a wavefront's rows each wait on their own chain of index reads, so a layer with many rows gets
    // four rows per wavefront (16 lanes, each walking several 16-byte pieces); measured on 54 k rows of 1 KB: 34 -> 25 us,
    // on 6 k rows: slower than one row per wavefront
    const int lg_cap = n_src >= 16384 ? 4 : 6;
    int lg = 0;
    while ((1 << lg) < pieces && lg < lg_cap) ++lg;
    const int gpb = BW_THREADS >> lg;
    int64_t blocks = fg_ceil_div(n_src, gpb);
    if (blocks > 256 * 16) blocks = 256 * 16;
    // with groups smaller than a wavefront: workgroups of their own for the positions with many incoming edges (one pass of
    // 64 positions per wavefront)
    const int sweep2 = lg < 6 ? (int)fg_ceil_div(n_src, 64 * (BW_THREADS / 64)) : 0;
    if (gcn)
        hipLaunchKernelGGL(aggregate_backward_kernel<true>, dim3((unsigned)(blocks + sweep2)), dim3(BW_THREADS), 0, st, (const char*)dx, n, d_in,
                           live_dev, hit_dev, row_start_dev, row_end_dev, t_start_dev, t_end_dev, t_row_dev, nnz, n_src, (char*)dh_src_dev,
                           dh_src_stride, lg, norms_src_dev, 16, sweep2);
    else
        hipLaunchKernelGGL(aggregate_backward_kernel<false>, dim3((unsigned)(blocks + sweep2)), dim3(BW_THREADS), 0, st, (const char*)dx, n, d_in,
                           live_dev, hit_dev, row_start_dev, row_end_dev, t_start_dev, t_end_dev, t_row_dev, nnz, n_src, (char*)dh_src_dev,
                           dh_src_stride, lg, norms_src_dev, 16, sweep2);
    FG_LAUNCH_CHECK("aggregate_backward_kernel");
    return FG_OK;
}

#define FG_LAYER_BACKWARD_ARGS                                                                                                      \
    dh_dev, dh_stride, h_dev, h_stride, n, rows_dev, n_rows_dev, max_rows, live_dev, hit_dev, row_start_dev, row_end_dev, t_start_dev, \
        t_end_dev, t_row_dev, nnz, n_src, d_in, d_out, W, dh_src_dev, dh_src_stride, norms_src_dev, ws_dev, ws_bytes, stream

extern "C" fg_status_t fg_layer_backward(const float* dh_dev, int64_t dh_stride, const float* h_dev, int64_t h_stride, int32_t n,
                                         const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                                         const uint8_t* live_dev, const uint8_t* hit_dev, const int32_t* row_start_dev,
                                         const int32_t* row_end_dev, const int32_t* t_start_dev, const int32_t* t_end_dev,
                                         const int32_t* t_row_dev, int64_t nnz, int32_t n_src, int32_t d_in, int32_t d_out,
                                         const float* W, float* dh_src_dev, int64_t dh_src_stride, float* norms_src_dev,
                                         void* ws_dev, size_t ws_bytes, void* stream) {
    return layer_backward_launch("fg_layer_backward", BW_SAGE_F32, FG_LAYER_BACKWARD_ARGS);
}

extern "C" fg_status_t fg_layer_backward_gcn(const float* dh_dev, int64_t dh_stride, const float* h_dev, int64_t h_stride, int32_t n,
                                             const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                                             const uint8_t* live_dev, const uint8_t* hit_dev, const int32_t* row_start_dev,
                                             const int32_t* row_end_dev, const int32_t* t_start_dev, const int32_t* t_end_dev,
                                             const int32_t* t_row_dev, int64_t nnz, int32_t n_src, int32_t d_in, int32_t d_out,
                                             const float* W, float* dh_src_dev, int64_t dh_src_stride, float* norms_src_dev,
                                             void* ws_dev, size_t ws_bytes, void* stream) {
    return layer_backward_launch("fg_layer_backward_gcn", BW_GCN_F32, FG_LAYER_BACKWARD_ARGS);
}

extern "C" fg_status_t fg_layer_backward_bf16(const float* dh_dev, int64_t dh_stride, const void* h_dev, int64_t h_stride, int32_t n,
                                              const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                                              const uint8_t* live_dev, const uint8_t* hit_dev, const int32_t* row_start_dev,
                                              const int32_t* row_end_dev, const int32_t* t_start_dev, const int32_t* t_end_dev,
                                              const int32_t* t_row_dev, int64_t nnz, int32_t n_src, int32_t d_in, int32_t d_out,
                                              const void* W, float* dh_src_dev, int64_t dh_src_stride, float* norms_src_dev,
                                              void* ws_dev, size_t ws_bytes, void* stream) {
    return layer_backward_launch("fg_layer_backward_bf16", BW_SAGE_BF16, FG_LAYER_BACKWARD_ARGS);
}
#undef FG_LAYER_BACKWARD_ARGS

// ---- weight gradients --------------------------------------------------------------------------------------
//
// dW = X^T . dz and db = column sums of dz over the computed rows, X[k, :] = [h_src[rows[k], :] ‖ agg[k, :]],
// dz[k, :] = dh[rows[k], :] * (h[rows[k], :] > 0). A contraction over the rows (K = tens of thousands) with a small
// result (2*d_in x d_out), so K is split over the workgroups: workgroup `chunk` multiplies its rows on the matrix
// cores and leaves a partial result, a second launch adds the partials up in fp64. Two kernels for the partial
// products: weight_grad_partial_x3_kernel (further down, the default: bf16 matrix instructions on three-way splits of
// both operands) and this one on the fp32 matrix instructions (operands beyond 4 GB, or asked for through the tuning key).
// Here both operands are read straight from global memory in the layout v_mfma_f32_32x32x2_f32 wants (for the two rows k, k+1 a
// lane supplies one element of row k + lane/32 per block), with no transposition and no LDS.
// A workgroup of 8 wavefronts (4 along M x 2 along N) owns a 256 x 256 tile of the result, a wavefront 64 x 128 of it as
// 2 x 4 blocks of 32 x 32. The blocks interleave: a lane's elements for the two row blocks are adjacent columns of X and
// those for the four column blocks adjacent columns of dz, so a pair of rows costs a lane one 8-byte and two 16-byte loads
// (dh and h) for 8 matrix instructions.
namespace {

constexpr int WG_THREADS = 512;
constexpr int WG_TILE = 256;
constexpr int WG_PAIRS = 3;  // pairs of rows whose loads are issued together

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(WG_THREADS) void weight_grad_partial_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, const char* __restrict__ agg, int64_t agg_stride,
    const char* __restrict__ dh, int64_t dh_stride, const char* __restrict__ h, int64_t h_stride, int n,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out,
    float* __restrict__ part_w, float* __restrict__ part_b) {
    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    const int M = 2 * d_in, N = d_out;
    const int chunk = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, kh = lane >> 5;
    const int wm = wave & 3, wn = wave >> 2;
    const int m_base = blockIdx.y * WG_TILE + wm * 64;
    const int n_base = blockIdx.z * WG_TILE + wn * 128;
    // the rows there are, split evenly over the chunks of the launch (whole batches per chunk)
    const int64_t per = (n_rows + gridDim.x - 1) / gridDim.x;
    const int64_t per_b = (per + 2 * WG_PAIRS - 1) / (2 * WG_PAIRS) * (2 * WG_PAIRS);
    const int64_t k_begin = (int64_t)chunk * per_b < n_rows ? (int64_t)chunk * per_b : n_rows;
    int64_t k_end = k_begin + per_b;
    if (k_end > n_rows) k_end = n_rows;

    // This lane's columns. A wavefront's 64 rows of the result are split over its two row blocks by parity and its 128
    // columns over its four column blocks modulo 4, so that a lane's operands for all blocks are adjacent in memory:
    // X[k][m_pair], X[k][m_pair + 1] (one 8-byte load) and dz[k][n_quad .. n_quad + 3] (16-byte loads).
    // Row l of result block i is then row m_base + 2*l + i, column l of result block j is column n_base + 4*l + j.
    const int m_pair = m_base + 2 * l32;
    const bool a_ok = m_pair < M;              // M is even: both columns exist or neither
    const bool a_self = m_pair < d_in;         // d_in is even: a pair never straddles the two panels
    const int a_col = a_ok ? (a_self ? m_pair : m_pair - d_in) : 0;
    const int n_quad = n_base + 4 * l32;
    const bool b_ok = n_quad < N;              // N is a multiple of 4
    const int b_col = b_ok ? n_quad : 0;
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    float colsum[4] = {0.f, 0.f, 0.f, 0.f};

    // the position of list entry k, or of entry k_begin where k is past the chunk (that entry exists whenever this is called)
    auto row_of = [&](int64_t kk) -> int32_t {
        const int64_t ks = kk < k_end ? kk : k_begin;
        return rows ? rows[ks] : (int32_t)ks;
    };
    // One batch = WG_PAIRS pairs of rows: 11 loads per pair and lane, then 8 matrix instructions per pair. Two batches are
    // kept in registers: while one is multiplied the loads of the next are in flight. The row positions are fetched one
    // batch further ahead so that the row loads do not wait for them.
    struct Batch {
        f32x2 a[WG_PAIRS];
        f32x4 g[WG_PAIRS], o[WG_PAIRS];
        bool ok[WG_PAIRS];
    };
    int32_t r_next[WG_PAIRS];
#pragma unroll
    for (int p = 0; p < WG_PAIRS; ++p) r_next[p] = k_begin < k_end ? row_of(k_begin + 2 * p + kh) : 0;
    auto load_batch = [&](int64_t k0, Batch& B) {  // all loads from a safe row where this lane has none; masks come later
#pragma unroll
        for (int p = 0; p < WG_PAIRS; ++p) {
            const int64_t kk = k0 + 2 * p + kh;
            const bool in = kk < k_end;
            const int64_t ks = in ? kk : k_begin;
            const int32_t r = r_next[p];
            r_next[p] = row_of(kk + 2 * WG_PAIRS);
            B.ok[p] = in && r >= 0 && r < n && r < n_src;
            const int64_t rs = B.ok[p] ? r : 0;
            const float* xs = (const float*)(h_src + rs * src_stride);
            const float* xa = (const float*)(agg + ks * agg_stride);
            B.a[p] = *(const f32x2*)((a_self ? xs : xa) + a_col);
            const float* gr = (const float*)(dh + rs * dh_stride);
            const float* hr = h ? (const float*)(h + rs * h_stride) : gr;
            B.g[p] = *(const f32x4*)(gr + b_col);
            B.o[p] = *(const f32x4*)(hr + b_col);
        }
    };
    auto multiply_batch = [&](Batch& B) {
#pragma unroll
        for (int p = 0; p < WG_PAIRS; ++p) {
#pragma unroll
            for (int i = 0; i < 2; ++i) B.a[p][i] = (B.ok[p] && a_ok) ? B.a[p][i] : 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool pass = B.ok[p] && b_ok && (h ? B.o[p][j] > 0.f : true);
                B.g[p][j] = pass ? B.g[p][j] : 0.f;
                colsum[j] += B.g[p][j];
            }
        }
#pragma unroll
        for (int p = 0; p < WG_PAIRS; ++p)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(B.a[p][i], B.g[p][j], acc[i][j], 0, 0, 0);
    };
    constexpr int64_t STEP = 2 * WG_PAIRS;
    Batch X, Y;
    if (k_begin < k_end) load_batch(k_begin, X);
    for (int64_t k0 = k_begin; k0 < k_end; k0 += 2 * STEP) {
        const bool second = k0 + STEP < k_end;            // uniform over the workgroup
        if (second) load_batch(k0 + STEP, Y);
        __builtin_amdgcn_sched_barrier(0);                // the next batch's loads are issued before this batch's arithmetic
        multiply_batch(X);
        if (k0 + 2 * STEP < k_end) load_batch(k0 + 2 * STEP, X);
        __builtin_amdgcn_sched_barrier(0);
        if (second) multiply_batch(Y);
    }
    // partial result of this chunk (zeros if the chunk lies beyond the rows there are)
    float* pw = part_w + (int64_t)chunk * M * N;
    // a lane's elements of the four column blocks are four adjacent columns of one row: one 16-byte store
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = m_base + 2 * (8 * (e >> 2) + 4 * kh + (e & 3)) + i;  // accumulator element e is block row 8*(e/4) + 4*kh + e%4
            const f32x4 v = {acc[i][0][e], acc[i][1][e], acc[i][2][e], acc[i][3][e]};
            if (m < M && b_ok) *(f32x4*)(pw + (int64_t)m * N + n_quad) = v;
        }
    if (blockIdx.y == 0 && wm == 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float s = colsum[j] + __shfl_xor(colsum[j], 32, 64);
            const int c = n_quad + j;
            if (kh == 0 && c < N) part_b[(int64_t)chunk * N + c] = s;
        }
    }
}

// The same partial products on the bf16 matrix cores. Every fp32 value is the exact sum of three bf16 values
// (x1 = bf16(x), x2 = bf16(x - x1), x3 = bf16(x - x1 - x2), nearest even), and the six products a_i * b_j with i + j <= 4
// (1-based; each exact in fp32) are kept: the dropped three are below 2^-24 of the product. v_mfma_f32_32x32x16_bf16 wants
// its contraction index contiguous in a lane, which for X^T . dz is the row index, so both operands go through LDS
// transposed: a step is 16 rows; thread (column c, group g) of the workgroup loads the 8 values X[k0 + 8g .. + 7][c] (each
// load coalesced over the columns), splits them and writes the three 16-byte fragments where the lane that needs them
// for (column c, k half g) reads them back with one LDS load: [term][g][column], conflict-free both ways. The same thread
// does the same for dz (mask applied to the loaded values, column sums for db kept in a register). Splitting is shared by
// the whole workgroup: 16 values per thread and step next to 48 matrix instructions per wavefront. Two LDS buffers, one
// barrier per step; the values of step s + 1 and the row positions of step s + 2 are in flight while step s is multiplied.
// A wavefront owns 64 x 128 of the 256 x 256 tile as before; fp32 sums within a slice, fp64 across the slices.
typedef unsigned int wu32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 wbf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 wbf16x2 __attribute__((ext_vector_type(2)));

constexpr int WX_STEP = 16;                          // rows per step: the K of one matrix instruction
constexpr int WX_FRAGS = 3 * 2 * WG_TILE;            // 16-byte fragments of one operand per step
constexpr size_t WX_LDS_BYTES = (size_t)2 * 2 * WX_FRAGS * 16;  // two operands, two buffers: 96 KB

// v[0..7] -> three fragments of eight bf16 (element j in half j % 2 of word j / 2)
__device__ __forceinline__ void wx_split8(const float* v, wu32x4& t1, wu32x4& t2, wu32x4& t3) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const f32x2 x = {v[2 * p], v[2 * p + 1]};
        const wbf16x2 b1 = __builtin_convertvector(x, wbf16x2);
        const unsigned int u1 = __builtin_bit_cast(unsigned int, b1);
        const f32x2 r1 = {x[0] - __uint_as_float(u1 << 16), x[1] - __uint_as_float(u1 & 0xFFFF0000u)};
        const wbf16x2 b2 = __builtin_convertvector(r1, wbf16x2);
        const unsigned int u2 = __builtin_bit_cast(unsigned int, b2);
        const f32x2 r2 = {r1[0] - __uint_as_float(u2 << 16), r1[1] - __uint_as_float(u2 & 0xFFFF0000u)};
        const wbf16x2 b3 = __builtin_convertvector(r2, wbf16x2);
        t1[p] = u1;
        t2[p] = u2;
        t3[p] = __builtin_bit_cast(unsigned int, b3);
    }
}

__global__ __launch_bounds__(WG_THREADS, 2) void weight_grad_partial_x3_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, const char* __restrict__ agg, int64_t agg_stride,
    const char* __restrict__ dh, int64_t dh_stride, const char* __restrict__ h, int64_t h_stride, int n,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out,
    float* __restrict__ part_w, float* __restrict__ part_b) {
    extern __shared__ __attribute__((aligned(16))) wu32x4 wx_lds[];   // [buffer][operand][term][group][column]
    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    const int M = 2 * d_in, N = d_out;
    const int chunk = blockIdx.x;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = wave & 3, wn = wave >> 2;
    const int m_tile = blockIdx.y * WG_TILE, n_tile = blockIdx.z * WG_TILE;
    // the rows there are, split evenly over the chunks of the launch (whole steps per chunk)
    const int64_t per = (n_rows + gridDim.x - 1) / gridDim.x;
    const int64_t per_b = (per + WX_STEP - 1) / WX_STEP * WX_STEP;
    const int64_t k_begin = (int64_t)chunk * per_b < n_rows ? (int64_t)chunk * per_b : n_rows;
    int64_t k_end = k_begin + per_b;
    if (k_end > n_rows) k_end = n_rows;
    const int n_steps = (int)((k_end - k_begin + WX_STEP - 1) / WX_STEP);

    // staging role of this thread: column pc of both tiles, rows 8 * pg .. 8 * pg + 7 of a step
    const int pc = t & (WG_TILE - 1), pg = t >> 8;
    const int xc = m_tile + pc;
    const bool x_ok = xc < M, x_self = xc < d_in;
    const int x_col = x_ok ? (x_self ? xc : xc - d_in) : 0;
    const int zc = n_tile + pc;
    const bool z_ok = zc < N;
    const int z_col = z_ok ? zc : 0;

    // The loaded values of one step wait in registers: they are requested a whole step (its matrix instructions, its
    // barrier) before they are split and written to LDS, the row positions one step earlier still.
    struct Vals {
        float xv[8], gv[8], ov[8];
        unsigned ok;     // bit e: row e exists
    };
    int32_t pos_next[8];
    float colsum = 0.f;
    // positions of the rows of step s (list entries k_begin + 16 s + 8 pg + e); an entry past the chunk reads entry k_begin
    auto load_positions = [&](int s) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t kk = k_begin + (int64_t)s * WX_STEP + 8 * pg + e;
            const int64_t ks = kk < k_end ? kk : k_begin;
            pos_next[e] = rows ? rows[ks] : (int32_t)ks;
        }
    };
    // values of step s from the positions loaded for it; rows that do not exist read row 0 / entry k_begin and count as zero
    auto load_values = [&](int s, Vals& V) {
        V.ok = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t kk = k_begin + (int64_t)s * WX_STEP + 8 * pg + e;
            const bool in = kk < k_end;
            const int64_t ks = in ? kk : k_begin;
            const int32_t r = pos_next[e];
            const bool ok = in && r >= 0 && r < n && r < n_src;
            V.ok |= ok ? (1u << e) : 0u;
            // byte offsets in 32 bits (the host checks that every operand is below 4 GB): one register per address
            const uint32_t rs = ok ? (uint32_t)r : 0u;
            const uint32_t x_off = x_self ? rs * (uint32_t)src_stride + 4u * (uint32_t)x_col
                                          : (uint32_t)ks * (uint32_t)agg_stride + 4u * (uint32_t)x_col;
            V.xv[e] = *(const float*)((x_self ? h_src : agg) + x_off);
            V.gv[e] = *(const float*)(dh + (rs * (uint32_t)dh_stride + 4u * (uint32_t)z_col));
            V.ov[e] = h ? *(const float*)(h + (rs * (uint32_t)h_stride + 4u * (uint32_t)z_col)) : 1.f;
        }
    };
    // mask, split and write the loaded step to buffer b
    auto stage = [&](int b, const Vals& V) {
        float xs8[8], zs8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool ok = (V.ok >> e) & 1u;
            xs8[e] = (ok && x_ok) ? V.xv[e] : 0.f;
            zs8[e] = (ok && z_ok && V.ov[e] > 0.f) ? V.gv[e] : 0.f;
            colsum += zs8[e];
        }
        wu32x4 a1, a2, a3, b1, b2, b3;
        wx_split8(xs8, a1, a2, a3);
        wx_split8(zs8, b1, b2, b3);
        wu32x4* X = wx_lds + (size_t)b * 2 * WX_FRAGS;
        wu32x4* Z = X + WX_FRAGS;
        X[(0 * 2 + pg) * WG_TILE + pc] = a1;
        X[(1 * 2 + pg) * WG_TILE + pc] = a2;
        X[(2 * 2 + pg) * WG_TILE + pc] = a3;
        Z[(0 * 2 + pg) * WG_TILE + pc] = b1;
        Z[(1 * 2 + pg) * WG_TILE + pc] = b2;
        Z[(2 * 2 + pg) * WG_TILE + pc] = b3;
    };

    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // one step out of buffer b: 48 matrix instructions per wavefront
    auto multiply = [&](int b) {
        const wu32x4* X = wx_lds + (size_t)b * 2 * WX_FRAGS;
        const wu32x4* Z = X + WX_FRAGS;
        wu32x4 ax[2][3];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int term = 0; term < 3; ++term) ax[mb][term] = X[(term * 2 + half) * WG_TILE + wm * 64 + mb * 32 + l32];
        // (X term, dz term) pairs, smallest products first
        constexpr int TA[6] = {2, 0, 1, 1, 0, 0};
        constexpr int TZ[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            wu32x4 bz[3];
#pragma unroll
            for (int term = 0; term < 3; ++term) bz[term] = Z[(term * 2 + half) * WG_TILE + wn * 128 + nb * 32 + l32];
#pragma unroll
            for (int e = 0; e < 6; ++e)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(wbf16x8, ax[mb][TA[e]]),
                                                                          __builtin_bit_cast(wbf16x8, bz[TZ[e]]), acc[mb][nb], 0, 0, 0);
        }
    };

    if (n_steps > 0) {      // uniform over the workgroup
        Vals V;
        load_positions(0);
        load_values(0, V);
        if (n_steps > 1) load_positions(1);
        stage(0, V);
        if (n_steps > 1) {
            load_values(1, V);
            if (n_steps > 2) load_positions(2);
        }
        __syncthreads();
        for (int s = 0; s < n_steps; ++s) {
            const int b = s & 1;
            // step s + 1 goes to the other buffer (last read a step ago, before the previous barrier), then the registers take
            // step s + 2, and step s is multiplied with those loads in flight
            if (s + 1 < n_steps) stage(b ^ 1, V);
            if (s + 2 < n_steps) {
                load_values(s + 2, V);
                if (s + 3 < n_steps) load_positions(s + 3);
            }
            __builtin_amdgcn_sched_barrier(0);
            multiply(b);
            __syncthreads();
        }
    }
    // partial result of this chunk (zeros if the chunk lies beyond the rows there are): accumulator element e of a block is
    // its row 8 * (e / 4) + 4 * half + e % 4, column l32
    float* pw = part_w + (int64_t)chunk * M * N;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = m_tile + wm * 64 + mb * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const int c = n_tile + wn * 128 + nb * 32 + l32;
                if (m < M && c < N) pw[(int64_t)m * N + c] = acc[mb][nb][e];
            }
        }
    if (blockIdx.y == 0) {      // column sums of dz: the two row groups of a column meet in LDS
        float* red = (float*)wx_lds;
        red[t] = colsum;
        __syncthreads();
        if (t < WG_TILE && z_ok) part_b[(int64_t)chunk * N + zc] = red[t] + red[t + WG_TILE];
    }
}

// dw[i] = sum over the chunks of part_w[chunk][i] in fp64. A workgroup owns 128 consecutive elements (32 lanes x 4) and
// splits the chunks over its 8 wavefront halves; db (the last workgroups) likewise.
constexpr int RED_GROUPS = BW_THREADS / 32;
__global__ __launch_bounds__(BW_THREADS) void weight_grad_reduce_kernel(const float* __restrict__ part_w,
                                                                        const float* __restrict__ part_b, int n_chunks,
                                                                        int64_t mn, int n_cols, int w_blocks,
                                                                        float* __restrict__ dw, float* __restrict__ db) {
    __shared__ double red[RED_GROUPS][32][4];
    const int tx = threadIdx.x & 31, g = threadIdx.x >> 5;
    const bool is_w = (int)blockIdx.x < w_blocks;
    const float* part = is_w ? part_w : part_b;
    const int64_t len = is_w ? mn : n_cols;  // both multiples of 4
    float* out = is_w ? dw : db;
    const int64_t i = ((int64_t)(is_w ? blockIdx.x : blockIdx.x - w_blocks) * 32 + tx) * 4;
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    if (i < len) {
        for (int c = g; c < n_chunks; c += 4 * RED_GROUPS) {
            f32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int cc = c + u * RED_GROUPS;
                v[u] = cc < n_chunks ? *(const f32x4*)(part + (int64_t)cc * len + i) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                s[0] += (double)v[u].x;
                s[1] += (double)v[u].y;
                s[2] += (double)v[u].z;
                s[3] += (double)v[u].w;
            }
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) red[g][tx][q] = s[q];
    __syncthreads();
    if (g == 0 && i < len && out) {
        double t[4] = {0.0, 0.0, 0.0, 0.0};
        for (int gg = 0; gg < RED_GROUPS; ++gg)
#pragma unroll
            for (int q = 0; q < 4; ++q) t[q] += red[gg][tx][q];
        const f32x4 o = {(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
        *(f32x4*)(out + i) = o;
    }
}

// Mixed precision: the weight gradients as a product on the bf16 matrix cores. Both operands of dW = X^T . dz are bf16 values
// (the rows of X as the forward product rounded them, dz rounded after the mask), so the contraction over the computed rows
// is a plain bf16 matrix product; the matrix instruction wants the contraction index contiguous, which for X^T . dz is the
// row index. This kernel writes both operands transposed, XT [2*d_in x Kp] and DZT [d_out x Kp] in bf16 (Kp = the bound on
// the rows rounded up to 64; zeros from the row count to the end of its block of 64), 64 x 64 tiles through LDS, reads and
// writes coalesced. The dz tiles also leave the column sums of the unrounded dz of their 64 rows (the bias gradient's
// partial sums; zeros for blocks beyond the rows there are).
constexpr int ST_TILE = 64;
__global__ __launch_bounds__(BW_THREADS) void weight_grad_stage_bf16_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, int src_code, const char* __restrict__ agg, int64_t agg_stride,
    const char* __restrict__ dh, int64_t dh_stride, const char* __restrict__ h, int64_t h_stride, int n,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out, int tiles_x,
    unsigned short* __restrict__ xt, unsigned short* __restrict__ dzt, int64_t kp, float* __restrict__ part_b) {
    __shared__ unsigned short tile[ST_TILE][ST_TILE + 2];
    __shared__ float sums[BW_THREADS / ST_TILE][ST_TILE];
    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    const int64_t k0 = (int64_t)blockIdx.x * ST_TILE;
    const bool is_x = (int)blockIdx.y < tiles_x;
    const int c0 = (is_x ? (int)blockIdx.y : (int)blockIdx.y - tiles_x) * ST_TILE;   // first column of X (of 2*d_in) or of dz
    const int n_cols = is_x ? 2 * d_in : d_out;
    const int tx = threadIdx.x & (ST_TILE - 1), ty = threadIdx.x / ST_TILE;          // 64 x 4
    const int c = c0 + tx;
    if (k0 >= n_rows) {      // nothing to stage: only the bias gradient's partial sums need their zeros
        if (!is_x && ty == 0 && c < d_out) part_b[(int64_t)blockIdx.x * d_out + c] = 0.f;
        return;
    }
    float colsum = 0.f;
    for (int rr = ty; rr < ST_TILE; rr += BW_THREADS / ST_TILE) {
        const int64_t k = k0 + rr;
        float v = 0.f;
        if (k < n_rows && c < n_cols) {
            const int32_t r = rows ? rows[k] : (int32_t)k;
            if (r >= 0 && r < n) {
                if (is_x) {
                    if (c < d_in) {
                        if (r < n_src) {
                            const char* row = h_src + (int64_t)r * src_stride;
                            v = src_code == FG_F32 ? ((const float*)row)[c]
                                : src_code == FG_F16 ? __half2float(__ushort_as_half(((const unsigned short*)row)[c]))
                                                     : bw_bf16_value(((const unsigned short*)row)[c]);
                        }
                    } else {
                        v = bw_bf16_value(((const unsigned short*)(agg + k * agg_stride))[c - d_in]);
                    }
                } else {
                    v = ((const float*)(dh + (int64_t)r * dh_stride))[c];
                    if (h && !(bw_bf16_value(((const unsigned short*)(h + (int64_t)r * h_stride))[c]) > 0.f)) v = 0.f;
                    colsum += v;
                }
            }
        }
        tile[rr][tx] = bw_bf16_bits(v);
    }
    if (!is_x) sums[ty][tx] = colsum;
    __syncthreads();
    if (!is_x && ty == 0 && c < d_out) {
        float t = 0.f;
#pragma unroll
        for (int q = 0; q < BW_THREADS / ST_TILE; ++q) t += sums[q][tx];
        part_b[(int64_t)blockIdx.x * d_out + c] = t;
    }
    unsigned short* out = is_x ? xt : dzt;
    for (int cc = ty; cc < ST_TILE; cc += BW_THREADS / ST_TILE)
        if (c0 + cc < n_cols) out[(int64_t)(c0 + cc) * kp + k0 + tx] = tile[tx][cc];
}

struct WgStage {
    int64_t kp;
    size_t dzt, part_b, total;
};
WgStage wg_stage_plan(int64_t max_rows, int64_t d_in, int64_t d_out) {
    WgStage p;
    p.kp = fg_ceil_div(max_rows > 0 ? max_rows : 1, ST_TILE) * ST_TILE;
    p.dzt = fg_align_up((size_t)(2 * d_in) * p.kp * 2, 256);
    p.part_b = p.dzt + fg_align_up((size_t)d_out * p.kp * 2, 256);
    p.total = p.part_b + fg_align_up((size_t)(p.kp / ST_TILE) * d_out * 4, 256);
    return p;
}

struct WgPlan {
    int n_chunks, rows_per_chunk, tiles_m, tiles_n;
    size_t part_b, total;
};
WgPlan wg_plan(int64_t max_rows, int64_t d_in, int64_t d_out) {
    WgPlan p;
    p.tiles_m = (int)fg_ceil_div(2 * d_in, WG_TILE);
    p.tiles_n = (int)fg_ceil_div(d_out, WG_TILE);
    int64_t chunks = 256 / (p.tiles_m * p.tiles_n);  // one workgroup per compute unit
    if (chunks < 1) chunks = 1;
    const int64_t by_rows = fg_ceil_div(max_rows > 0 ? max_rows : 1, 32);  // at least 32 rows per chunk (1024 rows: 40 -> 30 us against 64)
    if (chunks > by_rows) chunks = by_rows;
    int64_t per = fg_ceil_div(max_rows > 0 ? max_rows : 1, chunks);
    per = fg_ceil_div(per, 2 * WG_PAIRS) * 2 * WG_PAIRS;
    p.rows_per_chunk = (int)per;
    p.n_chunks = (int)fg_ceil_div(max_rows > 0 ? max_rows : 1, per);
    p.part_b = fg_align_up((size_t)p.n_chunks * 2 * d_in * d_out * 4, 256);
    p.total = p.part_b + fg_align_up((size_t)p.n_chunks * d_out * 4, 256);
    return p;
}

}  // namespace

extern "C" size_t fg_layer_backward_weights_workspace_bytes(int64_t max_rows, int32_t d_in, int32_t d_out) {
    if (max_rows < 0 || d_in <= 0 || d_out <= 0) return 0;
    return wg_plan(max_rows, d_in, d_out).total;
}

extern "C" fg_status_t fg_layer_backward_weights(const float* h_src_dev, int32_t n_src, int64_t src_stride, const float* agg_dev,
                                                 int64_t agg_stride, const float* dh_dev, int64_t dh_stride, const float* h_dev,
                                                 int64_t h_stride, int32_t n, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                                 int64_t max_rows, int32_t d_in, int32_t d_out, float* dw_dev, float* db_dev,
                                                 void* ws_dev, size_t ws_bytes, void* stream) {
    const char* who = "fg_layer_backward_weights";
    if (n < 0 || n_src < 0 || max_rows < 0 || d_in <= 0 || d_out <= 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: bad size (n %d, n_src %d, max_rows %lld, d_in %d, d_out %d)", who, n, n_src, (long long)max_rows, d_in, d_out);
    if (!dw_dev) FG_FAIL(FG_ERR_INVALID_ARG, "%s: dw_dev is NULL", who);
    if (d_out % 4) FG_FAIL(FG_ERR_SHAPE, "%s: d_out = %d must be a multiple of 4", who, d_out);
    if (((uintptr_t)dw_dev | (uintptr_t)db_dev) & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: dw_dev and db_dev must be 16-byte aligned", who);
    if (max_rows > 0 && n > 0 && n_src > 0 && (!h_src_dev || !agg_dev || !dh_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (src_stride < (int64_t)d_in * 4 || agg_stride < (int64_t)d_in * 4 || dh_stride < (int64_t)d_out * 4 || (h_dev && h_stride < (int64_t)d_out * 4))
        FG_FAIL(FG_ERR_SHAPE, "%s: a row stride is smaller than its row", who);
    if (d_in % 4) FG_FAIL(FG_ERR_SHAPE, "%s: d_in = %d must be a multiple of 4", who, d_in);
    if (((uintptr_t)h_src_dev | (uintptr_t)agg_dev | (uintptr_t)dh_dev | (uintptr_t)h_dev | (uintptr_t)src_stride | (uintptr_t)agg_stride |
         (uintptr_t)dh_stride | (uintptr_t)h_stride) & 15)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_src, agg, dh, h and their strides must be 16-byte aligned", who);
    const WgPlan P = wg_plan(max_rows, d_in, d_out);
    if (!ws_dev || ws_bytes < P.total) FG_FAIL(FG_ERR_SHAPE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes, P.total);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: the workspace must be 16-byte aligned", who);
    fg_clear_error();
    hipStream_t st = (hipStream_t)stream;
    float* part_w = (float*)ws_dev;
    float* part_b = (float*)((char*)ws_dev + P.part_b);
    // without rows (or without anything they could index) every chunk is empty and the partials are zeros
    const int64_t rows_bound = (n > 0 && n_src > 0) ? max_rows : 0;
    // the products on the bf16 matrix cores (three-way split of both operands) unless the fp32 instructions are asked for
    const int64_t forced = fg_tuning(FG_TUNE_LINEAR_TILE);
    // (its byte offsets are 32-bit: every operand has to end below 4 GB)
    const int64_t lim = (int64_t)1 << 32;
    const bool near = (int64_t)n_src * src_stride < lim && max_rows * agg_stride < lim && (int64_t)n * dh_stride < lim &&
                      (!h_dev || (int64_t)n * h_stride < lim);
    if (forced == 32 || forced == 64 || forced == 128 || !near)
        hipLaunchKernelGGL(weight_grad_partial_kernel, dim3((unsigned)P.n_chunks, (unsigned)P.tiles_m, (unsigned)P.tiles_n), dim3(WG_THREADS), 0, st,
                           (const char*)h_src_dev, n_src, src_stride, (const char*)agg_dev, agg_stride, (const char*)dh_dev, dh_stride,
                           (const char*)h_dev, h_stride, n, rows_dev, n_rows_dev, rows_bound, d_in, d_out, part_w, part_b);
    else
        hipLaunchKernelGGL(weight_grad_partial_x3_kernel, dim3((unsigned)P.n_chunks, (unsigned)P.tiles_m, (unsigned)P.tiles_n), dim3(WG_THREADS),
                           WX_LDS_BYTES, st, (const char*)h_src_dev, n_src, src_stride, (const char*)agg_dev, agg_stride, (const char*)dh_dev,
                           dh_stride, (const char*)h_dev, h_stride, n, rows_dev, n_rows_dev, rows_bound, d_in, d_out, part_w, part_b);
    FG_LAUNCH_CHECK("weight_grad_partial_kernel");
    const int64_t mn = (int64_t)2 * d_in * d_out;
    const int w_blocks = (int)fg_ceil_div(mn, 128), b_blocks = (int)fg_ceil_div(d_out, 128);
    hipLaunchKernelGGL(weight_grad_reduce_kernel, dim3((unsigned)(w_blocks + b_blocks)), dim3(BW_THREADS), 0, st, part_w, part_b, P.n_chunks,
                       mn, d_out, w_blocks, dw_dev, db_dev);
    FG_LAUNCH_CHECK("weight_grad_reduce_kernel");
    return FG_OK;
}

extern "C" size_t fg_layer_backward_weights_bf16_workspace_bytes(int64_t max_rows, int32_t d_in, int32_t d_out) {
    if (max_rows < 0 || d_in <= 0 || d_out <= 0) return 0;
    return wg_stage_plan(max_rows, d_in, d_out).total;
}

extern "C" fg_status_t fg_layer_backward_weights_bf16(const void* h_src_dev, int32_t n_src, int64_t src_stride, fg_dtype_t src_dtype,
                                                      const void* agg_dev, int64_t agg_stride, const float* dh_dev, int64_t dh_stride,
                                                      const void* h_dev, int64_t h_stride, int32_t n, const int32_t* rows_dev,
                                                      const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in, int32_t d_out,
                                                      float* dw_dev, float* db_dev, void* ws_dev, size_t ws_bytes, void* stream) {
    const char* who = "fg_layer_backward_weights_bf16";
    if (n < 0 || n_src < 0 || max_rows < 0 || d_in <= 0 || d_out <= 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: bad size (n %d, n_src %d, max_rows %lld, d_in %d, d_out %d)", who, n, n_src, (long long)max_rows, d_in, d_out);
    if (!dw_dev) FG_FAIL(FG_ERR_INVALID_ARG, "%s: dw_dev is NULL", who);
    if (src_dtype != FG_F32 && src_dtype != FG_F16 && src_dtype != FG_BF16) FG_FAIL(FG_ERR_DTYPE, "%s: h_src must be fp32, fp16 or bf16", who);
    const int64_t src_esz = src_dtype == FG_F32 ? 4 : 2;
    if (d_in % 8 || d_out % 8) FG_FAIL(FG_ERR_SHAPE, "%s: d_in = %d and d_out = %d must be multiples of 8", who, d_in, d_out);
    if (((uintptr_t)dw_dev | (uintptr_t)db_dev) & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: dw_dev and db_dev must be 16-byte aligned", who);
    if (max_rows > 0 && n > 0 && n_src > 0 && (!h_src_dev || !agg_dev || !dh_dev)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (src_stride < (int64_t)d_in * src_esz || agg_stride < (int64_t)d_in * 2 || dh_stride < (int64_t)d_out * 4 || (h_dev && h_stride < (int64_t)d_out * 2))
        FG_FAIL(FG_ERR_SHAPE, "%s: a row stride is smaller than its row", who);
    if (((uintptr_t)h_src_dev | (uintptr_t)agg_dev | (uintptr_t)dh_dev | (uintptr_t)h_dev | (uintptr_t)src_stride | (uintptr_t)agg_stride |
         (uintptr_t)dh_stride | (uintptr_t)h_stride) & 3)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_src, agg, dh, h and their strides must be 4-byte aligned", who);
    const WgStage P = wg_stage_plan(max_rows, d_in, d_out);
    if (!ws_dev || ws_bytes < P.total) FG_FAIL(FG_ERR_SHAPE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes, P.total);
    if ((uintptr_t)ws_dev & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: the workspace must be 16-byte aligned", who);
    fg_clear_error();
    hipStream_t st = (hipStream_t)stream;
    unsigned short* xt = (unsigned short*)ws_dev;
    unsigned short* dzt = (unsigned short*)((char*)ws_dev + P.dzt);
    float* part_b = (float*)((char*)ws_dev + P.part_b);
    // without rows (or without anything they could index) nothing is staged and the product below is over nothing
    const int64_t rows_bound = (n > 0 && n_src > 0) ? max_rows : 0;
    const int tiles_k = (int)(P.kp / ST_TILE), tiles_x = (int)fg_ceil_div(2 * d_in, ST_TILE), tiles_z = (int)fg_ceil_div(d_out, ST_TILE);
    hipLaunchKernelGGL(weight_grad_stage_bf16_kernel, dim3((unsigned)tiles_k, (unsigned)(tiles_x + tiles_z)), dim3(BW_THREADS), 0, st,
                       (const char*)h_src_dev, n_src, src_stride, (int)src_dtype, (const char*)agg_dev, agg_stride, (const char*)dh_dev,
                       dh_stride, (const char*)h_dev, h_stride, n, rows_dev, n_rows_dev, rows_bound, d_in, d_out, tiles_x, xt, dzt, P.kp,
                       part_b);
    FG_LAUNCH_CHECK("weight_grad_stage_bf16_kernel");
    // dW [2*d_in x d_out] = XT . DZT^T: the forward kernel with XT's rows as its rows (both halves of its K from the one
    // matrix), DZT as the transposed weights, K = the rows there are (a count in device memory, or the bound)
    const int64_t half_k = P.kp / 2;
    const int64_t* k_limit = nullptr;
    // the count the K loop stops at must be min(*n_rows_dev, rows_bound): the staging kernel zero-fills up to the end of
    // that block of 64; with a host-side bound only, the whole of Kp is valid (zeros beyond the rows)
    if (n_rows_dev && rows_bound == max_rows) k_limit = n_rows_dev;
    if (rows_bound == 0) {      // nothing staged: dW = 0 without touching the (unwritten) operands
        fg_status_t rc = fg_launch_fill_i32((int32_t*)dw_dev, (int64_t)2 * d_in * d_out, 0, st);
        if (rc != FG_OK) return rc;
    } else {
        fg_status_t rc = fg_launch_linear_bf16(xt, 2 * d_in, P.kp * 2, FG_BF16, xt + half_k, P.kp * 2, nullptr, nullptr, 2 * d_in,
                                               (int32_t)half_k, d_out, dzt, nullptr, 0, dw_dev, 2 * d_in, (int64_t)d_out * 4, FG_F32, st,
                                               true, k_limit);
        if (rc != FG_OK) return rc;
    }
    if (db_dev) {
        const int b_blocks = (int)fg_ceil_div(d_out, 128);
        hipLaunchKernelGGL(weight_grad_reduce_kernel, dim3((unsigned)b_blocks), dim3(BW_THREADS), 0, st, part_b, part_b, tiles_k, (int64_t)0,
                           d_out, 0, dw_dev, db_dev);
        FG_LAUNCH_CHECK("weight_grad_reduce_kernel");
    }
    return FG_OK;
}
