// bf16 variant of the dense layer update (phi of Eq. 1): bf16 operands on v_mfma_f32_32x32x16_bf16, fp32
// accumulation, bias and ReLU in fp32, output rounded once to bf16 (hidden layers) or kept in fp32 (last layer).
// Used by the workload whose raw features are fp16 and whose embeddings, weights and cache rows are bf16.
//
// K is walked in steps of 64 = four 16-deep MFMA sub-steps. Both operands sit in LDS with k contiguous (rows of 72
// halfwords: 16-byte aligned, conflict-free for the 16-byte operand reads): a lane's MFMA operand is one 16-byte LDS
// read. A is gathered on the fly (own rows from h_src at the listed positions, converted from fp16 to bf16 if needed;
// mean rows from the compact agg array). The weights come either transposed, [N x K], and are then loaded and written
// to LDS like the rows of A, or row-major [K x N]: then a thread reads two adjacent k rows x 8 columns and writes the
// eight (k, k+1) pairs transposed as 32-bit words.
#include <hip/hip_fp16.h>

#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int HB_K = 64;
constexpr int LDH = HB_K + 8;  // halfwords per LDS row: 144 bytes, so that the 16-byte reads of neighbouring rows fall on different banks

__device__ __forceinline__ unsigned int f32_to_bf16_bits(float f) {
    const unsigned int b = __float_as_uint(f);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

// eight fp16 values (packed in 4 words) -> eight bf16 values, each rounded to nearest even (the packed conversion
// instruction of this chip: three instructions per pair)
__device__ __forceinline__ u32x4 f16x8_to_bf16x8(u32x4 v) {
    const f32x8 f = __builtin_convertvector(__builtin_bit_cast(f16x8, v), f32x8);
    return __builtin_bit_cast(u32x4, __builtin_convertvector(f, bf16x8));
}

// HB_M x HB_N: the workgroup's output tile (128 x 128 or 64 x 64). The small tile has four wavefronts as 2 x 2, each
// owning one block of 32 x 32; it gives layers with few rows enough workgroups to hide the latency of the operand loads
// behind each other. The 128 x 128 tile has eight wavefronts as 2 x 4, each owning
// 64 x 32 of it: at under 128 registers a lane, two such workgroups (four wavefronts per SIMD) share a compute unit, and
// it is wavefronts waiting on different things that keep the matrix cores fed.
// W_NK: the weights are given transposed, [N x K] with k contiguous: their tile is then loaded and written to LDS like
// the rows of A, 16 bytes at a time, with nothing to reshuffle.
//
// Pipeline: the operands of K step s + 2 are on their way from memory to registers and those of step s + 1 on their way
// from registers to the second LDS buffer while step s is multiplied out of the first: a load has two steps of
// arithmetic to arrive in, and one barrier per step suffices (a buffer is written two steps after it was last read,
// with the barrier of the step in between). fp16 inputs are converted when they are written to LDS, not when they are
// loaded, so the loads stay in flight.
// Every load is issued unconditionally from an address that is valid whatever the row and k are (a row that does not
// exist reads the tile's first row, a k beyond K reads k = 0). Rows and columns that do not exist need no zeroing: an
// output depends on its own row of A and its own column of W only, and theirs are never written. Only the k values
// beyond K of a last, partial step are written to LDS as zeros (both operands, so that nothing non-finite meets a zero).
constexpr size_t hb_lds_bytes(int hb_m, int hb_n) { return (size_t)2 * (hb_m + hb_n) * LDH * 2 + (size_t)hb_m * 8; }

constexpr int hb_waves(int hb_m, int hb_n) { return hb_m * hb_n >= 128 * 128 ? 8 : 4; }

template <bool SRC_F16, bool OUT_BF16, int HB_M, int HB_N, bool W_NK>
__global__ __launch_bounds__(64 * hb_waves(HB_M, HB_N), hb_waves(HB_M, HB_N) == 8 ? 4 : 2) void linear_bf16_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, const char* __restrict__ agg, int64_t agg_stride,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out,
    const unsigned short* __restrict__ W, const float* __restrict__ bias, int relu, char* __restrict__ h_out, int n_out,
    int64_t out_stride, int n_tiles, const int64_t* __restrict__ k_limit_dev, const int32_t* __restrict__ src_ids) {
    extern __shared__ __attribute__((aligned(16))) unsigned short hb_lds[];
    constexpr int HB_WAVES = hb_waves(HB_M, HB_N), HB_THREADS = 64 * HB_WAVES;
    constexpr int STAGE = (HB_M + HB_N) * LDH;    // halfwords per buffer: A rows, then the columns of W
    int32_t* row_of = (int32_t*)(hb_lds + 2 * STAGE);   // output position of each row of the tile, -1: none
    int32_t* src_of = row_of + HB_M;                     // the row of h_src with its own features: the position, or src_ids[position]

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
        int32_t r = -1, s = -1;
        if (g < n_rows) {
            r = rows ? rows[g] : (int32_t)g;
            if (r < 0 || r >= n_out) r = -1;
            if (r >= 0) s = src_ids ? src_ids[r] : r;
            if (s < 0 || s >= n_src) r = s = -1;
        }
        row_of[t] = r;
        src_of[t] = s;
    }
    __syncthreads();

    constexpr int A_PIECES = HB_K / 8;               // 8-element pieces of a row per k step
    constexpr int A_ROWS = HB_THREADS / A_PIECES;    // rows covered by one pass of the workgroup
    constexpr int A_PASSES = HB_M / A_ROWS;
    // W as [K x N]: a thread takes 8 columns of two adjacent k rows; as [N x K]: 8 k values of one column, like A
    constexpr int B_PIECES = HB_N / 8;               // 8-column pieces of a row of the W tile
    constexpr int B_PAIRS = HB_THREADS / B_PIECES;   // pairs of k rows covered by one pass of the workgroup
    constexpr int B_PASSES = W_NK ? HB_N / A_ROWS : (HB_K / 2) / B_PAIRS;
    constexpr int B_REGS = W_NK ? B_PASSES : 2 * B_PASSES;
    const int a_kc = t % A_PIECES;   // which 8-element piece of the k step
    const int a_m = t / A_PIECES;    // rows a_m + A_ROWS * i
    // (the k pair runs fastest over the lanes: their 32-bit transposed writes then fall on different LDS banks)
    const int b_kp = t % B_PAIRS;    // k pairs b_kp + B_PAIRS * q: rows 2 kp, 2 kp + 1
    const int b_nc = t / B_PAIRS;    // columns 8 b_nc .. 8 b_nc + 7
    // per thread: the positions of its A rows and, relative to the tile's first mean row / first weight column (which always
    // exist), the rows of its other loads: 32 bits each; a row or column that does not exist reads the first one instead
    int32_t a_row[A_PASSES], agg_rel[A_PASSES];
    const int32_t r_first = src_of[0];          // the tile's first row exists (m0 < n_rows), its position may still be out of range
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
        const int m = a_m + A_ROWS * i;
        const int32_t r = src_of[m];
        a_row[i] = r >= 0 ? r : (r_first >= 0 ? r_first : 0);
        agg_rel[i] = m0 + m < n_rows ? m : 0;   // list entries below the count lie within the caller's max_rows
    }
    const char* agg_first = agg + m0 * agg_stride;
    const bool b_col_ok = (n0 + 8 * b_nc) < d_out;
    const unsigned short* w_col = W + (b_col_ok ? n0 + 8 * b_nc : 0);        // [K x N]
    const unsigned short* w_first = W + (int64_t)n0 * K;                      // [N x K]: column n0 (n0 < d_out)
    int32_t w_rel[W_NK ? B_PASSES : 1];
    if constexpr (W_NK) {
#pragma unroll
        for (int i = 0; i < B_PASSES; ++i) w_rel[i] = n0 + a_m + A_ROWS * i < d_out ? a_m + A_ROWS * i : 0;
    }

    struct Regs {
        u32x4 a[A_PASSES], b[B_REGS];
    };
    auto load_step = [&](int k0, Regs& R) {
        const int ka = k0 + 8 * a_kc;
        const bool own = ka < d_in;
        const int64_t a_off = (int64_t)(ka < K ? (own ? ka : ka - d_in) : 0) * 2;
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i) {
            const char* from = own ? h_src + (int64_t)a_row[i] * src_stride : agg_first + (int64_t)agg_rel[i] * agg_stride;
            R.a[i] = *(const u32x4*)(from + a_off);
        }
        if constexpr (W_NK) {
            const int kw = ka < K ? ka : 0;
#pragma unroll
            for (int i = 0; i < B_PASSES; ++i) R.b[i] = *(const u32x4*)(w_first + (int64_t)w_rel[i] * K + kw);
        } else {
#pragma unroll
            for (int q = 0; q < B_PASSES; ++q)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int kb = k0 + 2 * (b_kp + B_PAIRS * q) + i;
                    R.b[2 * q + i] = *(const u32x4*)(w_col + (int64_t)(kb < K ? kb : 0) * d_out);
                }
        }
    };
    const bool k_tail = (K % HB_K) != 0;     // the last step is partial
    auto store_step = [&](int k0, const Regs& R, int buf) {
        unsigned short* As = hb_lds + buf * STAGE;
        unsigned short* Bt = As + HB_M * LDH;
        const bool convert = SRC_F16 && (k0 + 8 * a_kc) < d_in;   // this piece comes from the fp16 rows
        const bool a_k_ok = (k0 + 8 * a_kc) < K;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i) {
            const int m = a_m + A_ROWS * i;
            u32x4 v = convert ? f16x8_to_bf16x8(R.a[i]) : R.a[i];
            if (k_tail) v = a_k_ok ? v : zero;
            *(u32x4*)(As + m * LDH + 8 * a_kc) = v;
        }
        if constexpr (W_NK) {
#pragma unroll
            for (int i = 0; i < B_PASSES; ++i) {
                const int c = a_m + A_ROWS * i;
                u32x4 v = R.b[i];
                if (k_tail) v = a_k_ok ? v : zero;
                *(u32x4*)(Bt + c * LDH + 8 * a_kc) = v;
            }
        } else {
#pragma unroll
            for (int p = 0; p < B_PASSES; ++p) {
                const int kp = b_kp + B_PAIRS * p;      // k values 2 kp, 2 kp + 1: word kp & 3 of chunk kp >> 2
                const bool k0_ok = !k_tail || (k0 + 2 * kp) < K, k1_ok = !k_tail || (k0 + 2 * kp + 1) < K;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    // word q of each loaded row holds columns 2q (low half) and 2q + 1 (high half)
                    const unsigned int lo = k0_ok ? R.b[2 * p][q] : 0u, hi = k1_ok ? R.b[2 * p + 1][q] : 0u;
                    const int c = 8 * b_nc + 2 * q;
                    *(unsigned int*)(Bt + c * LDH + 2 * kp) = (lo & 0xFFFFu) | (hi << 16);
                    *(unsigned int*)(Bt + (c + 1) * LDH + 2 * kp) = (lo >> 16) | (hi & 0xFFFF0000u);
                }
            }
        }
    };

    const int lane = t & 63, wave = t >> 6;
    constexpr int WN = HB_WAVES / 2;                           // wavefronts along N (two along M)
    constexpr int MB = HB_M / 64, NB = HB_N / (32 * WN);       // 32 x 32 blocks per wavefront
    const int wm = (wave / WN) * (HB_M / 2), wn = (wave % WN) * (HB_N / WN);
    const int l32 = lane & 31, half = lane >> 5;

    f32x16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
    // the operands of sub-step kk + 1 are read from LDS while the matrix instructions of sub-step kk run
    auto multiply_step = [&](int buf) {
        const unsigned short* As = hb_lds + buf * STAGE;
        const unsigned short* Bt = As + HB_M * LDH;
        bf16x8 av[2][MB], bv[2][NB];
        auto read_operands = [&](int kk, int set) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int m = wm + mb * 32 + l32;
                av[set][mb] = *(const bf16x8*)(As + m * LDH + 16 * kk + 8 * half);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int c = wn + nb * 32 + l32;
                bv[set][nb] = *(const bf16x8*)(Bt + c * LDH + 16 * kk + 8 * half);
            }
        };
        // with four wavefronts per SIMD the others cover the LDS latency and the second set of operand registers is not worth its cost
        constexpr bool AHEAD = HB_WAVES == 4;
        if (AHEAD) read_operands(0, 0);
#pragma unroll
        for (int kk = 0; kk < HB_K / 16; ++kk) {
            if (AHEAD) {
                if (kk + 1 < HB_K / 16) read_operands(kk + 1, (kk + 1) & 1);
            } else {
                read_operands(kk, 0);
            }
            const int set = AHEAD ? (kk & 1) : 0;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[set][mb], bv[set][nb], acc[mb][nb], 0, 0, 0);
        }
    };

    // k_limit_dev (optional): only the first *k_limit_dev values of k count (the caller guarantees zeros from there to the end
    // of that K step), so the K loop stops there: the contraction length is then a count in device memory
    int nk = (K + HB_K - 1) / HB_K;
    if (k_limit_dev) {
        const int64_t lim = *k_limit_dev;
        const int64_t steps = lim <= 0 ? 0 : (lim + HB_K - 1) / HB_K;
        if (steps < nk) nk = (int)steps;
    }
    Regs R0, R1;
    load_step(0, R0);
    if (nk > 1) load_step(HB_K, R1);
    store_step(0, R0, 0);
    if (nk > 2) load_step(2 * HB_K, R0);
    __syncthreads();
    for (int s = 0; s < nk; s += 2) {
        // step s out of buffer 0; step s + 1 goes to buffer 1, step s + 3 sets out from memory
        if (s + 1 < nk) {
            store_step((s + 1) * HB_K, R1, 1);
            if (s + 3 < nk) load_step((s + 3) * HB_K, R1);
        }
        multiply_step(0);
        __syncthreads();
        if (s + 1 >= nk) break;
        if (s + 2 < nk) {
            store_step((s + 2) * HB_K, R0, 0);
            if (s + 4 < nk) load_step((s + 4) * HB_K, R0);
        }
        multiply_step(1);
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
                                  fg_dtype_t out_dtype, hipStream_t st, bool w_nk, const int64_t* k_limit_dev,
                                  const int32_t* src_ids_dev) {
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
    if (max_rows == 0 || n_src == 0 || n_out == 0) return FG_OK;     // no row can be in range
    // tile by the number of workgroups the bound on the rows gives (the rows there are may be a fraction of it): the large
    // tile once it fills most of the chip, else the small one, whose many workgroups hide each other's load latency
    const int64_t t128 = fg_ceil_div(max_rows, 128) * fg_ceil_div(d_out, 128);
    int tile = t128 >= 192 ? 128 : 64;
    const int64_t forced = fg_tuning(FG_TUNE_LINEAR_TILE);     // 1128: 128 x 128, 1064: 64 x 64
    if (forced == 1128) tile = 128;
    if (forced == 1064) tile = 64;
    const int ny = (int)fg_ceil_div(d_out, tile);
    const int64_t m_tiles = fg_ceil_div(max_rows, tile);
    const unsigned grid = (unsigned)(fg_ceil_div(m_tiles, 8) * 8 * ny);
#define FG_LB4(F16, OBF, TM, TN, NK)                                                                                       \
    hipLaunchKernelGGL((linear_bf16_kernel<F16, OBF, TM, TN, NK>), dim3(grid), dim3(64 * hb_waves(TM, TN)), hb_lds_bytes(TM, TN), st, \
                       (const char*)h_src, n_src, src_stride, (const char*)agg, agg_stride, rows_dev, n_rows_dev, max_rows, \
                       d_in, d_out, (const unsigned short*)W, bias, relu, (char*)h_out, n_out, out_stride, ny, k_limit_dev, src_ids_dev)
#define FG_LB3(F16, OBF, TM, TN)         \
    do {                                 \
        if (w_nk)                        \
            FG_LB4(F16, OBF, TM, TN, true);  \
        else                             \
            FG_LB4(F16, OBF, TM, TN, false); \
    } while (0)
#define FG_LB(F16, OBF)                    \
    do {                                   \
        if (tile == 128)                   \
            FG_LB3(F16, OBF, 128, 128);    \
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
#undef FG_LB4
    FG_LAUNCH_CHECK("linear_bf16_kernel");
    return FG_OK;
}
