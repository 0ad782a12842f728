// bf16 variant of the dense layer update (phi of Eq. 1): bf16 operands on v_mfma_f32_32x32x16_bf16, fp32
// accumulation, bias and ReLU in fp32, output rounded once to bf16 (hidden layers) or kept in fp32 (last layer).
// Used by the workload whose raw features are fp16 and whose embeddings, weights and cache rows are bf16.
//
// A workgroup of four wavefronts owns a 128 x 128 output tile, each wavefront a 64 x 64 quadrant (2 x 2 MFMA
// blocks). K is walked in steps of 64 = four 16-deep MFMA sub-steps. Both operands sit in LDS with k contiguous
// (rows of 72 halfwords: 16-byte aligned, conflict-free for the 16-byte operand reads): a lane's MFMA operand
// is one 16-byte LDS read. A is gathered on the fly (own rows from h_src at the listed positions, converted
// from fp16 to bf16 if needed; mean rows from the compact agg array). W is row-major [K x N] in memory, so each
// thread reads two adjacent k rows x 8 columns and writes the eight (k, k+1) pairs transposed as 32-bit words.
#include <hip/hip_fp16.h>

#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int HB_K = 64;
constexpr int LDH = HB_K + 8;  // halfwords per LDS row
constexpr int HB_THREADS = 256;

__device__ __forceinline__ unsigned int f32_to_bf16_bits(float f) {
    const unsigned int b = __float_as_uint(f);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float f16_bits_to_f32(unsigned int h) {
    return __half2float(__ushort_as_half((unsigned short)h));
}

// eight fp16 values (packed in 4 words) -> eight bf16 values, each rounded to nearest even
__device__ __forceinline__ u32x4 f16x8_to_bf16x8(u32x4 v) {
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned int w = v[i];
        o[i] = f32_to_bf16_bits(f16_bits_to_f32(w & 0xFFFFu)) | (f32_to_bf16_bits(f16_bits_to_f32(w >> 16)) << 16);
    }
    return o;
}

// HB_M x HB_N: the workgroup's output tile (128 x 128, 64 x 128 or 64 x 64): four wavefronts as 2 x 2, each owning
// (HB_M / 64) x (HB_N / 64) blocks of 32 x 32. Smaller tiles give layers with few rows enough workgroups to hide the
// latency of the operand loads behind each other.
template <bool SRC_F16, bool OUT_BF16, int HB_M, int HB_N>
__global__ __launch_bounds__(HB_THREADS, 2) void linear_bf16_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, const char* __restrict__ agg, int64_t agg_stride,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out,
    const unsigned short* __restrict__ W, const float* __restrict__ bias, int relu, char* __restrict__ h_out, int n_out,
    int64_t out_stride, int n_tiles) {
    __shared__ __attribute__((aligned(16))) unsigned short As[HB_M * LDH];
    __shared__ __attribute__((aligned(16))) unsigned short Bt[HB_N * LDH];
    __shared__ int32_t row_of[HB_M];

    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    // column tiles of one row tile share an XCD (and its L2), as in the fp32 kernel
    const int xcd = blockIdx.x & 7;
    const int j = blockIdx.x >> 3;
    const int64_t m0 = ((int64_t)(j / n_tiles) * 8 + xcd) * HB_M;
    if (m0 >= n_rows) return;
    const int n0 = (j % n_tiles) * HB_N;
    const int t = threadIdx.x;
    const int K = 2 * d_in;

    if (t < HB_M) {
        const int64_t g = m0 + t;
        int32_t r = -1;
        if (g < n_rows) {
            r = rows ? rows[g] : (int32_t)g;
            if (r < 0 || r >= n_src || r >= n_out) r = -1;
        }
        row_of[t] = r;
    }
    __syncthreads();

    constexpr int A_PIECES = HB_K / 8;               // 8-element pieces of a row per k step
    constexpr int A_ROWS = HB_THREADS / A_PIECES;    // rows covered by one pass of the workgroup
    constexpr int A_PASSES = HB_M / A_ROWS;
    constexpr int B_PAIRS = HB_K / 2;                // pairs of k rows per k step
    constexpr int B_COLS = HB_THREADS / B_PAIRS * 8; // columns covered by one pass
    constexpr int B_PASSES = HB_N / B_COLS;
    const int a_kc = t % A_PIECES;   // which 8-element piece of the k step
    const int a_m = t / A_PIECES;    // rows a_m + A_ROWS * i
    const int b_kp = t % B_PAIRS;    // k pair (2 b_kp, 2 b_kp + 1)
    const int b_nc = t / B_PAIRS;    // columns 8 b_nc + B_COLS * q .. + 7
    const char* a_self[A_PASSES];
    const char* a_agg[A_PASSES];
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
        const int m = a_m + A_ROWS * i;
        const int32_t r = row_of[m];
        a_self[i] = r >= 0 ? h_src + (int64_t)r * src_stride : nullptr;
        a_agg[i] = r >= 0 ? agg + (m0 + m) * agg_stride : nullptr;
    }
    bool b_col_ok[B_PASSES];
#pragma unroll
    for (int q = 0; q < B_PASSES; ++q) b_col_ok[q] = (n0 + B_COLS * q + 8 * b_nc) < d_out;

    u32x4 ra[A_PASSES], rb[B_PASSES][2];
    auto load_step = [&](int k0) {
        const int ka = k0 + 8 * a_kc;
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (a_self[i] && ka < K) {
                if (ka < d_in) {
                    v = *(const u32x4*)(a_self[i] + (int64_t)ka * 2);
                    if (SRC_F16) v = f16x8_to_bf16x8(v);
                } else {
                    v = *(const u32x4*)(a_agg[i] + (int64_t)(ka - d_in) * 2);
                }
            }
            ra[i] = v;
        }
#pragma unroll
        for (int q = 0; q < B_PASSES; ++q)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int kb = k0 + 2 * b_kp + i;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (b_col_ok[q] && kb < K) v = *(const u32x4*)(W + (int64_t)kb * d_out + n0 + B_COLS * q + 8 * b_nc);
                rb[q][i] = v;
            }
    };
    auto store_step = [&]() {
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i) *(u32x4*)(As + (a_m + A_ROWS * i) * LDH + 8 * a_kc) = ra[i];
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // word q of each row holds columns 2q (low half) and 2q + 1 (high half)
                const unsigned int lo = rb[p][0][q], hi = rb[p][1][q];
                const int c = B_COLS * p + 8 * b_nc + 2 * q;
                *(unsigned int*)(Bt + c * LDH + 2 * b_kp) = (lo & 0xFFFFu) | (hi << 16);
                *(unsigned int*)(Bt + (c + 1) * LDH + 2 * b_kp) = (lo >> 16) | (hi & 0xFFFF0000u);
            }
    };

    const int lane = t & 63, wave = t >> 6;
    constexpr int MB = HB_M / 64, NB = HB_N / 64;  // 32 x 32 blocks per wavefront
    const int wm = (wave >> 1) * (HB_M / 2), wn = (wave & 1) * (HB_N / 2);
    const int l32 = lane & 31, half = lane >> 5;

    f32x16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    const int nk = (K + HB_K - 1) / HB_K;
    load_step(0);
    for (int step = 0; step < nk; ++step) {
        store_step();
        __syncthreads();
        if (step + 1 < nk) load_step((step + 1) * HB_K);
#pragma unroll
        for (int kk = 0; kk < HB_K / 16; ++kk) {
            bf16x8 av[MB], bv[NB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) av[mb] = *(const bf16x8*)(As + (wm + mb * 32 + l32) * LDH + 16 * kk + 8 * half);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) bv[nb] = *(const bf16x8*)(Bt + (wn + nb * 32 + l32) * LDH + 16 * kk + 8 * half);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[mb], bv[nb], acc[mb][nb], 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator element i of a 32x32 block is row 8*(i/4) + 4*half + i%4, column l32
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int c = n0 + wn + nb * 32 + l32;
        if (c >= d_out) continue;
        const float bvv = bias ? bias[c] : 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = wm + mb * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                const int32_t r = row_of[m];
                if (r < 0) continue;
                float v = acc[mb][nb][i] + bvv;
                if (relu) v = v > 0.f ? v : 0.f;
                if (OUT_BF16)
                    *(unsigned short*)(h_out + (int64_t)r * out_stride + (int64_t)c * 2) = (unsigned short)f32_to_bf16_bits(v);
                else
                    *(float*)(h_out + (int64_t)r * out_stride + (int64_t)c * 4) = v;
            }
        }
    }
}

}  // namespace

fg_status_t fg_launch_linear_bf16(const void* h_src, int32_t n_src, int64_t src_stride, fg_dtype_t in_dtype,
                                  const void* agg, int64_t agg_stride, const int32_t* rows_dev,
                                  const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in, int32_t d_out, const void* W,
                                  const float* bias, int32_t relu, void* h_out, int32_t n_out, int64_t out_stride,
                                  fg_dtype_t out_dtype, hipStream_t st) {
    if (in_dtype != FG_F16 && in_dtype != FG_BF16) FG_FAIL(FG_ERR_DTYPE, "fg_linear: bf16 weights need fp16 or bf16 inputs");
    if (out_dtype != FG_BF16 && out_dtype != FG_F32) FG_FAIL(FG_ERR_DTYPE, "fg_linear: bf16 weights give bf16 or fp32 outputs");
    if (d_in % 8 || d_out % 8) FG_FAIL(FG_ERR_SHAPE, "fg_linear: d_in = %d and d_out = %d must be multiples of 8 for 16-bit types", d_in, d_out);
    const int osz = out_dtype == FG_F32 ? 4 : 2;
    if (src_stride < (int64_t)d_in * 2 || agg_stride < (int64_t)d_in * 2 || out_stride < (int64_t)d_out * osz)
        FG_FAIL(FG_ERR_SHAPE, "fg_linear: a row stride is smaller than its row");
    if (((uintptr_t)h_src | (uintptr_t)agg | (uintptr_t)W | (uintptr_t)src_stride | (uintptr_t)agg_stride) & 15)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_linear: h_src, agg, W and the input strides must be 16-byte aligned");
    if (((uintptr_t)h_out | (uintptr_t)out_stride) & (uintptr_t)(osz - 1) || ((uintptr_t)bias & 3))
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_linear: h_out, its stride and bias must be aligned to their element size");
    fg_clear_error();
    if (max_rows == 0) return FG_OK;
    // tile by the number of workgroups the bound on the rows gives (the rows there are may be a fraction of it)
    const int64_t t128 = fg_ceil_div(max_rows, 128) * fg_ceil_div(d_out, 128);
    const int tm = t128 >= 512 ? 128 : 64;
    const int tn = (t128 >= 512 || fg_ceil_div(max_rows, 64) * fg_ceil_div(d_out, 128) >= 512) ? 128 : 64;
    const int ny = (int)fg_ceil_div(d_out, tn);
    const int64_t m_tiles = fg_ceil_div(max_rows, tm);
    const unsigned grid = (unsigned)(fg_ceil_div(m_tiles, 8) * 8 * ny);
#define FG_LB3(F16, OBF, TM, TN)                                                                                          \
    hipLaunchKernelGGL((linear_bf16_kernel<F16, OBF, TM, TN>), dim3(grid), dim3(HB_THREADS), 0, st, (const char*)h_src,    \
                       n_src, src_stride, (const char*)agg, agg_stride, rows_dev, n_rows_dev, max_rows, d_in, d_out,        \
                       (const unsigned short*)W, bias, relu, (char*)h_out, n_out, out_stride, ny)
#define FG_LB(F16, OBF)                    \
    do {                                   \
        if (tm == 128)                     \
            FG_LB3(F16, OBF, 128, 128);    \
        else if (tn == 128)                \
            FG_LB3(F16, OBF, 64, 128);     \
        else                               \
            FG_LB3(F16, OBF, 64, 64);      \
    } while (0)
    if (in_dtype == FG_F16) {
        if (out_dtype == FG_BF16) FG_LB(true, true); else FG_LB(true, false);
    } else {
        if (out_dtype == FG_BF16) FG_LB(false, true); else FG_LB(false, false);
    }
#undef FG_LB
#undef FG_LB3
    FG_LAUNCH_CHECK("linear_bf16_kernel");
    return FG_OK;
}
