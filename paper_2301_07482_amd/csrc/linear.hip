// fg_linear: h_out[r,:] = act([h_src[r,:] ‖ agg[k,:]] . W + bias) for r = rows[k]: the dense update phi of
// Eq. 1 for GraphSAGE-mean, the only dense contraction on the path, on the matrix cores.
//
// fp32 path: v_mfma_f32_32x32x2_f32. A workgroup of four wavefronts owns a (32*WM) x 64 output tile: WM = 4
// stacks the wavefronts along M (each 32 x 64, two MFMA blocks), WM = 2 arranges them 2 x 2 (each 32 x 32) for
// layers with few rows. Register use is kept low enough for three workgroups per compute unit, so that one
// workgroup's matrix instructions overlap another's loads. The A operand is never materialised: its first
// d_in columns are read from h_src at the listed positions and the last d_in from the compact agg array,
// 16 bytes at a time, through LDS. K is walked in steps of 32; inside a step the two half-wavefronts of an
// MFMA take k = s and k = 16 + s (s = 0..15), which lets every lane fetch its 16 A values as four 16-byte
// LDS reads (the sum over k does not care about the order). Global loads of the next step are issued
// before the MFMAs of the current one.
//
// Accuracy: a single fp32 accumulator over K = 512 products drifts by a few 1e-6 of the row scale, which is
// the whole error budget of the path (1e-5). Each 32-wide K step therefore starts from a zero fp32
// accumulator (small partial sums, small rounding steps) and is folded into an fp64 running sum on the
// vector ALU, two instructions per output element and step next to 16 matrix instructions; bias, ReLU and
// the single rounding to fp32 happen from the fp64 sum.
#include "common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BN = 64;
constexpr int KC = 32;  // k values per fp32 accumulation chunk (one fp64 fold per chunk)
constexpr int LDB = BN + 4;
constexpr int LIN_THREADS = 256;

// The row of h_src that holds the own features of position r: r itself, or src_ids[r] where the caller reads them straight
// from a table by row number (fg_linear_ids). -1 where there is no such row.
__device__ __forceinline__ int32_t own_row(const int32_t* __restrict__ src_ids, int32_t r, int n_src) {
    if (r < 0) return -1;
    const int32_t s = src_ids ? src_ids[r] : r;
    return (s < 0 || s >= n_src) ? -1 : s;
}

template <int WM, int BK>
__global__ __launch_bounds__(LIN_THREADS, 3) void linear_f32_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, const char* __restrict__ agg, int64_t agg_stride,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out,
    const float* __restrict__ W, const float* __restrict__ bias, int relu, char* __restrict__ h_out, int n_out,
    int64_t out_stride, int n_tiles, const int32_t* __restrict__ src_ids) {
    constexpr int BM = 32 * WM;
    constexpr int WN = 4 / WM;          // wavefronts along N
    constexpr int NB = BN / (32 * WN);  // 32-wide MFMA blocks per wavefront
    constexpr int LDA = BK + 4;  // floats; keeps 16-byte alignment and spreads rows over banks
    constexpr int A_LOADS = BM * BK / 4 / LIN_THREADS;
    constexpr int B_LOADS = BK * BN / 4 / LIN_THREADS;
    constexpr int A_CHUNKS = BK / 4;                 // 16-byte pieces per A row and step
    constexpr int A_ROWS = LIN_THREADS / A_CHUNKS;   // rows covered by one pass of the workgroup
    constexpr int B_ROWS = LIN_THREADS / 16;         // k rows covered by one pass of the workgroup
    __shared__ __attribute__((aligned(16))) float As[BM * LDA];
    __shared__ __attribute__((aligned(16))) float Bs[BK * LDB];
    __shared__ int32_t row_of[BM], src_of[BM];

    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2. The column tiles of one row
    // tile read the same A rows, so they are given consecutive slots of ONE XCD: id -> (xcd, j), row tile
    // (j / n_tiles) * 8 + xcd, column tile j % n_tiles. A then comes from HBM once instead of once per column tile.
    const int xcd = blockIdx.x & 7;
    const int j = blockIdx.x >> 3;
    const int64_t m0 = ((int64_t)(j / n_tiles) * 8 + xcd) * BM;
    if (m0 >= n_rows) return;
    const int n0 = (j % n_tiles) * BN;
    const int t = threadIdx.x;
    const int K = 2 * d_in;

    if (t < BM) {
        const int64_t g = m0 + t;
        int32_t r = -1, s = -1;
        if (g < n_rows) {
            r = rows ? rows[g] : (int32_t)g;
            if (r < 0 || r >= n_out) r = -1;
            s = own_row(src_ids, r, n_src);
            if (s < 0) r = -1;
        }
        row_of[t] = r;
        src_of[t] = s;
    }
    __syncthreads();

    // this thread's share of the global -> LDS traffic per step
    const int a_kc = t % A_CHUNKS;  // which 16-byte piece of the BK-wide k step
    const int a_m = t / A_CHUNKS;   // rows a_m + A_ROWS i
    const int b_nc = t & 15;        // which 16-byte piece of the 64-wide n tile
    const int b_k = t >> 4;         // k rows b_k + B_ROWS i
    // loads are unconditional (dummy address + select) so that the compiler can count the outstanding prefetch
    const float* a_self[A_LOADS];
    const float* a_agg[A_LOADS];
    bool a_ok[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int m = a_m + A_ROWS * i;
        const int32_t r = row_of[m];
        a_ok[i] = r >= 0;
        a_self[i] = (const float*)(h_src + (r >= 0 ? (int64_t)src_of[m] * src_stride : 0));
        a_agg[i] = (const float*)(agg + (r >= 0 ? (m0 + m) * agg_stride : 0));
    }
    const bool b_col_ok = (n0 + 4 * b_nc) < d_out;
    const int b_col = b_col_ok ? n0 + 4 * b_nc : 0;

    f32x4 ra[A_LOADS], rb[B_LOADS];
    auto load_step = [&](int k0) {
        const int ka = k0 + 4 * a_kc;
        // nothing here may touch the loaded values (a select would make the wavefront wait for the load on the
        // spot and undo the prefetch): out-of-range pieces are zeroed when they are written to LDS
        const int kac = ka < K ? ka : 0;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const float* p = kac < d_in ? a_self[i] + kac : a_agg[i] + (kac - d_in);
            ra[i] = *(const f32x4*)p;
        }
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) {
            const int kb = k0 + b_k + B_ROWS * i;
            rb[i] = *(const f32x4*)(W + (int64_t)(kb < K ? kb : 0) * d_out + b_col);
        }
    };
    auto store_step = [&](int k0) {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        const bool ka_ok = k0 + 4 * a_kc < K;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) *(f32x4*)(As + (a_m + A_ROWS * i) * LDA + 4 * a_kc) = (a_ok[i] && ka_ok) ? ra[i] : z;
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            *(f32x4*)(Bs + (b_k + B_ROWS * i) * LDB + 4 * b_nc) = (b_col_ok && k0 + b_k + B_ROWS * i < K) ? rb[i] : z;
    };

    const int lane = t & 63, wave = t >> 6;
    const int wm = (wave / WN) * 32, wn = (wave % WN) * 32 * NB;
    const int l32 = lane & 31, half = lane >> 5;

    double sum[NB][16];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) sum[b][i] = 0.0;

    const int nk = (K + BK - 1) / BK;
    load_step(0);
    for (int step = 0; step < nk; ++step) {
        store_step(step * BK);
        __syncthreads();
        load_step((step + 1) * BK);  // beyond K: reads a valid dummy address, zeroed at the LDS store
        // keep the prefetch ahead of the matrix instructions (the scheduler would otherwise sink it next to its use)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int hs = 0; hs < BK / KC; ++hs) {  // one fp32 accumulation chunk of 32 k values at a time
            f32x4 av[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) av[q] = *(const f32x4*)(As + (wm + l32) * LDA + KC * hs + 16 * half + 4 * q);
            f32x16 acc[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const float a = av[s >> 2][s & 3];
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const float bv = Bs[(KC * hs + 16 * half + s) * LDB + wn + 32 * b + l32];
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc[b], 0, 0, 0);
                }
            }
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) sum[b][i] += (double)acc[b][i];
        }
        __syncthreads();
    }

    // epilogue: accumulator element i of a 32x32 block is row 8*(i/4) + 4*half + i%4, column l32
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int c = n0 + wn + nb * 32 + l32;
        if (c >= d_out) continue;
        const double bv = bias ? (double)bias[c] : 0.0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = wm + 8 * (i >> 2) + 4 * half + (i & 3);
            const int32_t r = row_of[m];
            if (r < 0) continue;
            float v = (float)(sum[nb][i] + bv);
            if (relu) v = v > 0.f ? v : 0.f;
            *(float*)(h_out + (int64_t)r * out_stride + (int64_t)c * 4) = v;
        }
    }
}

// ---- panel variant: no barrier and no LDS on the A side (d_in a multiple of 32, a 32-column panel of W <= 64 KB) ------
//
//   * a workgroup (8 wavefronts) owns one 32-column panel of W, copies it to LDS once and synchronises once;
//   * a task is a 32-row block of the output times that panel; the wavefronts of the workgroups that own the
//     panel take row blocks round-robin and run them independently of each other;
//   * the A operand needs no LDS: with the k order used here (half-wavefront h takes k = 16h + s) a lane's 16
//     values of a K step are 64 contiguous bytes of its own row, loaded straight from memory one step ahead into
//     one of two register buffers. The loads are unconditional, their values are not touched before the matrix
//     instructions use them, and a scheduling barrier pins them ahead of the current step's matrix instructions:
//     a branch around a load, a select on its value, or the scheduler sinking it next to its use each turn the
//     prefetch into a full memory round trip per step. A row past the end reads row 0 instead (rows of a product
//     are independent and its results are never stored);
//   * B values are LDS broadcasts of one row of the panel per half-wavefront.
// Workgroups of the panels that share a row block have ids congruent mod 8 (same XCD): A comes from HBM once and
// from that XCD's L2 for the other panels.
constexpr int PL_THREADS = 512;
constexpr int PL_WAVES = PL_THREADS / 64;
constexpr int PL_BN = 32;

__global__ __launch_bounds__(PL_THREADS, 4) void linear_f32_panel_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, const char* __restrict__ agg, int64_t agg_stride,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out,
    const float* __restrict__ W, const float* __restrict__ bias, int relu, char* __restrict__ h_out, int n_out,
    int64_t out_stride, int n_panels, int n_groups, const int32_t* __restrict__ src_ids) {
    extern __shared__ __attribute__((aligned(16))) float panel[];  // [K][32]
    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    const int K = 2 * d_in;
    const int nk = K / KC, nk_self = d_in / KC;
    const int t = threadIdx.x;
    const int xcd = blockIdx.x & 7;
    const int j = blockIdx.x >> 3;
    const int n0 = (j % n_panels) * PL_BN;
    const int group = (j / n_panels) * 8 + xcd;
    const int64_t n_blocks = (n_rows + 31) >> 5;
    if (group >= n_blocks) return;  // uniform over the workgroup, before the barrier

    for (int q = t; q < K * 8; q += PL_THREADS) {
        const int k = q >> 3, c4 = (q & 7) * 4;
        const f32x4 v = *(const f32x4*)(W + (int64_t)k * d_out + (n0 + c4 < d_out ? n0 + c4 : 0));
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        *(f32x4*)(panel + k * PL_BN + c4) = n0 + c4 < d_out ? v : z;
    }
    __syncthreads();

    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int c = n0 + l32;
    const double bv = (bias && c < d_out) ? (double)bias[c] : 0.0;
    const float* bcol = panel + 16 * half * PL_BN + l32;

    // destination row of this lane in row block rb (-1: past the end or out of range) and, in s, the row of its own features
    auto row_of_block = [&](int64_t rb, int32_t& s) -> int32_t {
        const int64_t g = rb * 32 + l32;
        int32_t r = -1;
        s = -1;
        if (rb < n_blocks && g < n_rows) {
            r = rows ? rows[g] : (int32_t)g;
            if (r < 0 || r >= n_out) r = -1;
            s = own_row(src_ids, r, n_src);
            if (s < 0) r = -1;
        }
        return r;
    };
    const int64_t stride = (int64_t)n_groups * PL_WAVES;
    int64_t rb = group + (int64_t)n_groups * wave;
    if (rb >= n_blocks) return;
    int32_t s, s_next;
    int32_t r = row_of_block(rb, s);
    int32_t r_next = row_of_block(rb + stride, s_next);
    const float* a_self = (const float*)(h_src + (r >= 0 ? (int64_t)s * src_stride : 0)) + 16 * half;
    const float* a_agg = (const float*)(agg + (r >= 0 ? (rb * 32 + l32) * agg_stride : 0)) + 16 * half;
    f32x4 a0[4], a1[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) a0[q] = *(const f32x4*)(a_self + 4 * q);  // step 0 of the first task
    for (; rb < n_blocks; rb += stride) {
        // the row of the task after next is fetched now, and the next task's first K step during this task's last
        // one, so that the matrix instructions of consecutive tasks follow each other without a memory round trip
        int32_t s_after;
        const int32_t r_after = row_of_block(rb + 2 * stride, s_after);
        double sum[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) sum[i] = 0.0;
        auto compute = [&](int step, const f32x4* a) {
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
            const float* brow = bcol + step * KC * PL_BN;
#pragma unroll
            for (int s = 0; s < 16; ++s)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s >> 2][s & 3], brow[s * PL_BN], acc, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 16; ++i) sum[i] += (double)acc[i];
        };
        // nk = 2 * (d_in / 32) is even: both halves of the loop body run unconditionally (a condition around the
        // second one lets the compiler sink its loads into the conditional block, next to their use)
        for (int step = 0; step < nk; step += 2) {
            {
                const int s1 = step + 1;
                const float* p = s1 < nk_self ? a_self + s1 * KC : a_agg + (s1 - nk_self) * KC;
#pragma unroll
                for (int q = 0; q < 4; ++q) a1[q] = *(const f32x4*)(p + 4 * q);
            }
            __builtin_amdgcn_sched_barrier(0);
            compute(step, a0);
            {
                const int s2 = step + 2;
                const float* nxt = (const float*)(h_src + (r_next >= 0 ? (int64_t)s_next * src_stride : 0)) + 16 * half;
                const float* cur = s2 < nk_self ? a_self + s2 * KC : a_agg + (s2 < nk ? s2 - nk_self : 0) * KC;
                const float* p = s2 < nk ? cur : nxt;  // after the last step: step 0 of the next task (or a valid dummy)
#pragma unroll
                for (int q = 0; q < 4; ++q) a0[q] = *(const f32x4*)(p + 4 * q);
            }
            __builtin_amdgcn_sched_barrier(0);
            compute(step + 1, a1);
        }
        // accumulator element i is row 8*(i/4) + 4*half + i%4 of the block, column l32 of the panel
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = 8 * (i >> 2) + 4 * half + (i & 3);
            const int32_t rr = __shfl(r, m, 64);  // lane m (< 32) holds the destination row of block row m; all lanes active
            if (rr < 0 || c >= d_out) continue;
            float v = (float)(sum[i] + bv);
            if (relu) v = v > 0.f ? v : 0.f;
            *(float*)(h_out + (int64_t)rr * out_stride + (int64_t)c * 4) = v;
        }
        r = r_next;
        s = s_next;
        r_next = r_after;
        s_next = s_after;
        a_self = (const float*)(h_src + (r >= 0 ? (int64_t)s * src_stride : 0)) + 16 * half;
        a_agg = (const float*)(agg + (r >= 0 ? ((rb + stride) * 32 + l32) * agg_stride : 0)) + 16 * half;
    }
}

// The panel kernel with every fp32 product formed on the bf16 matrix cores. An fp32 value is the exact sum of three
// bf16 values (8 + 8 + 8 significand bits: x1 = bf16(x), x2 = bf16(x - x1), x3 = bf16(x - x1 - x2), each rounded to
// nearest even), so a*w = sum of a_i*w_j; the six terms with i + j <= 4 are kept (each exact in fp32), the three
// dropped ones are below 2^-26 |a*w|. Twelve v_mfma_f32_32x32x16_bf16 (six terms, two groups of 16 k) replace the
// sixteen v_mfma_f32_32x32x2_f32 of a 32-wide K chunk at 3/8 of their matrix-core time; accumulation is unchanged
// (fp32 inside a chunk, chunks folded into fp64). W is split once per workgroup while its panel is copied to
// LDS, stored as ready-made 16-byte B fragments; A is split in registers by the wavefront that loaded it, and a
// wavefront of the NB = 2 variant uses its split for two 32-column blocks.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr int X3_LIST = 8;                                  // tasks whose rows a wavefront lists ahead in LDS
constexpr int X3_LIST_BYTES = PL_WAVES * X3_LIST * 32 * 4;  // the lists of a workgroup (twice that with src_ids)

// v[0..7] -> three fragments of eight bf16 (element j in half j % 2 of word j / 2)
__device__ __forceinline__ void split8(const float* v, u32x4& t1, u32x4& t2, u32x4& t3) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const f32x2 x = {v[2 * p], v[2 * p + 1]};
        const bf16x2 b1 = __builtin_convertvector(x, bf16x2);
        const unsigned int u1 = __builtin_bit_cast(unsigned int, b1);
        const f32x2 r1 = {x[0] - __uint_as_float(u1 << 16), x[1] - __uint_as_float(u1 & 0xFFFF0000u)};
        const bf16x2 b2 = __builtin_convertvector(r1, bf16x2);
        const unsigned int u2 = __builtin_bit_cast(unsigned int, b2);
        const f32x2 r2 = {r1[0] - __uint_as_float(u2 << 16), r1[1] - __uint_as_float(u2 & 0xFFFF0000u)};
        const bf16x2 b3 = __builtin_convertvector(r2, bf16x2);
        t1[p] = u1;
        t2[p] = u2;
        t3[p] = __builtin_bit_cast(unsigned int, b3);
    }
}

// RAGGED: d_in is a multiple of 4 but not of 32. Each half of the operand is then walked as if it were d_pad = d_in rounded
// up to 32 wide: the k values from d_in to d_pad have zero weights in the panel, and the 16-byte pieces of a row that would
// lie there are read from 16 bytes of zeros instead (a piece lies wholly inside or wholly outside the row's d_in values).
__device__ __attribute__((aligned(16))) float x3_zero[4];

template <int NB, bool RAGGED>
__global__ __launch_bounds__(PL_THREADS, 2) void linear_f32x3_panel_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, const char* __restrict__ agg, int64_t agg_stride,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out,
    const float* __restrict__ W, const float* __restrict__ bias, int relu, char* __restrict__ h_out, int n_out,
    int64_t out_stride, int n_panels, int n_groups, int near_out, const int32_t* __restrict__ src_ids) {
    constexpr int BNW = PL_BN * NB;
    extern __shared__ __attribute__((aligned(16))) u32x4 bfrag[];  // [3 terms][K / 8 groups of k][BNW columns]
    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    const int d_pad = RAGGED ? (d_in + KC - 1) / KC * KC : d_in;
    const int K = 2 * d_pad;      // the contraction length as it is walked
    const int nk = K / KC, nk_self = d_pad / KC;
    const int ngr = K / 8;
    const int t = threadIdx.x;
    const int xcd = blockIdx.x & 7;
    const int j = blockIdx.x >> 3;
    const int n0 = (j % n_panels) * BNW;
    const int group = (j / n_panels) * 8 + xcd;
    const int64_t n_blocks = (n_rows + 31) >> 5;
    if (group >= n_blocks) return;  // uniform over the workgroup, before the barrier

    // group gi = (chunk * 2 + m) * 2 + half holds k = 32 * chunk + 16 * half + 8 * m + (0..7): the eight k values that
    // half-wavefront `half` feeds to matrix instruction m of the chunk. A thread takes a block of 8 k x 4 columns of W:
    // eight 16-byte loads, all issued before the first value is used (one memory round trip per pass, and the layers
    // of the workloads need a single pass), then the four columns' fragments.
    for (int q = t; q < ngr * (BNW / 4); q += PL_THREADS) {
        const int c4 = (q % (BNW / 4)) * 4, gi = q / (BNW / 4);
        const int k0 = 32 * (gi >> 2) + 16 * (gi & 1) + 8 * ((gi >> 1) & 1);
        const bool in = n0 + c4 < d_out;      // d_out is a multiple of 4: the four columns exist together
        const float* wp = W + (in ? n0 + c4 : 0);
        f32x4 w4[8];
        bool k_in[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {     // walked k -> row of W: the second half starts at d_in; padding rows read row 0
            const int kp = k0 + e, hf = (RAGGED && kp >= d_pad) ? 1 : 0, kk = kp - hf * d_pad;
            k_in[e] = !RAGGED || kk < d_in;
            const int wrow = RAGGED ? (k_in[e] ? hf * d_in + kk : 0) : kp;
            w4[e] = *(const f32x4*)(wp + (int64_t)wrow * d_out);
        }
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = (in && k_in[e]) ? w4[e][cc] : 0.f;
            u32x4 t1, t2, t3;
            split8(v, t1, t2, t3);
            bfrag[(0 * ngr + gi) * BNW + c4 + cc] = t1;
            bfrag[(1 * ngr + gi) * BNW + c4 + cc] = t2;
            bfrag[(2 * ngr + gi) * BNW + c4 + cc] = t3;
        }
    }
    __syncthreads();

    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    double bv[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int c = n0 + nb * 32 + l32;
        bv[nb] = (bias && c < d_out) ? (double)bias[c] : 0.0;
    }
    // The destination / source rows of a wavefront's next X3_LIST tasks are kept in LDS (behind the fragments): lane l32's
    // row of task t at rowlist[t * 32 + l32], -1 for a row past the end or out of range. Reading them costs no wait on
    // global memory: a global load of a row index in the middle of a task would make the wavefront wait for everything
    // it has in flight (the A values fetched ahead, the previous task's stores), since those complete in order.
    // With src_ids a second list holds the rows of h_src the own features come from (without: the same rows, one list).
    int32_t* rowlist = (int32_t*)(bfrag + 3 * ngr * BNW) + wave * (X3_LIST * 32);
    int32_t* srclist = src_ids ? rowlist + PL_WAVES * (X3_LIST * 32) : rowlist;
    auto row_raw = [&](int64_t rbx) -> int32_t {      // unconditional load: clamped index, a valid dummy address without a list
        int64_t g = rbx * 32 + l32;
        g = g < n_rows ? g : n_rows - 1;  // n_rows >= 1 here
        const int32_t* src = rows ? rows + g : (const int32_t*)h_src;
        return *src;
    };
    auto row_decode = [&](int32_t raw, int64_t rbx) -> int32_t {
        const int64_t g = rbx * 32 + l32;
        int32_t r = rows ? raw : (int32_t)g;
        if (rbx >= n_blocks || g >= n_rows || r < 0 || r >= n_out || (!src_ids && r >= n_src)) r = -1;
        return r;
    };
    const int64_t stride = (int64_t)n_groups * PL_WAVES;
    for (int64_t rb0 = group + (int64_t)n_groups * wave; rb0 < n_blocks; rb0 += X3_LIST * stride) {
        {
            int32_t raw[X3_LIST];
#pragma unroll
            for (int q = 0; q < X3_LIST; ++q) raw[q] = row_raw(rb0 + q * stride);
#pragma unroll
            for (int q = 0; q < X3_LIST; ++q) raw[q] = row_decode(raw[q], rb0 + q * stride);
            if (src_ids) {      // second round: the table rows of those positions (position 0 exists: n_out >= 1)
                int32_t sraw[X3_LIST];
#pragma unroll
                for (int q = 0; q < X3_LIST; ++q) sraw[q] = src_ids[raw[q] >= 0 ? raw[q] : 0];
#pragma unroll
                for (int q = 0; q < X3_LIST; ++q) {
                    if (raw[q] < 0 || sraw[q] < 0 || sraw[q] >= n_src) raw[q] = sraw[q] = -1;
                    srclist[q * 32 + l32] = sraw[q];
                }
            }
#pragma unroll
            for (int q = 0; q < X3_LIST; ++q) rowlist[q * 32 + l32] = raw[q];   // both halves write the same value
        }
        int32_t r = rowlist[l32], s = srclist[l32];
        const float* a_self = (const float*)(h_src + (r >= 0 ? (int64_t)s * src_stride : 0)) + 16 * half;
        const float* a_agg = (const float*)(agg + (r >= 0 ? (rb0 * 32 + l32) * agg_stride : 0)) + 16 * half;
        // the four 16-byte pieces of chunk `c` of one half of a row (base = that half's first value + 16 * half)
        auto load_chunk = [&](const float* base, int c, f32x4* a) {
            const float* p = base + c * KC;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool there = !RAGGED || c * KC + 16 * half + 4 * q < d_in;
                a[q] = *(const f32x4*)(there ? p + 4 * q : (const float*)x3_zero);
            }
        };
        f32x4 a0[4], a1[4];
        load_chunk(a_self, 0, a0);  // step 0 of the first task of the list
        for (int tk = 0; tk < X3_LIST; ++tk) {
            const int64_t rb = rb0 + tk * stride;
            if (rb >= n_blocks) break;
            // the row of the next task: its first K step is fetched during this task's last one (the last task of a
            // list fetches row 0 instead, and the next list starts with a fetch of its own)
            const int32_t r_next = tk + 1 < X3_LIST ? rowlist[(tk + 1) * 32 + l32] : -1;
            const int32_t s_next = tk + 1 < X3_LIST ? srclist[(tk + 1) * 32 + l32] : -1;
            // Two fp32 accumulators per column block, kept across the whole K range: `big` takes the products of the two
            // leading bf16 terms, `small` the five products that are 2^-8 and 2^-16 of those. What limits an fp32
            // running sum is the rounding of the sum itself at every accumulation step; with the leading term alone
            // `big` is rounded once per 16 k values (a sixth of the steps), and the roundings of `small` are 2^-8 of
            // that. Modelled and measured error: that of folding every 32 k values into fp64 (the output's own
            // rounding dominates), with none of the fold's vector work and half its registers.
            f32x16 big[NB], small[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i) big[nb][i] = small[nb][i] = 0.f;
            auto compute = [&](int step, const f32x4* a) {
                float av[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) av[q] = a[q >> 2][q & 3];
                u32x4 A[3][2];  // [term][m]
                split8(av, A[0][0], A[1][0], A[2][0]);
                split8(av + 8, A[0][1], A[1][1], A[2][1]);
                // (A term, W term) pairs of the small products, smallest first; the leading pair (0, 0) goes to `big`
                constexpr int TA[5] = {2, 0, 1, 1, 0};
                constexpr int TW[5] = {0, 2, 1, 0, 1};
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    u32x4 f[NB][3];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int term = 0; term < 3; ++term)
                            f[nb][term] = bfrag[term * ngr * BNW + ((step * 2 + m) * 2 + half) * BNW + nb * 32 + l32];
                    // the accumulator chains alternate, so that consecutive matrix instructions never depend on each other
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        big[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[0][m]),
                                                                          __builtin_bit_cast(bf16x8, f[nb][0]), big[nb], 0, 0, 0);
#pragma unroll
                    for (int e = 0; e < 5; ++e)
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            small[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[TA[e]][m]),
                                                                                __builtin_bit_cast(bf16x8, f[nb][TW[e]]), small[nb], 0, 0, 0);
                }
            };
            for (int step = 0; step < nk; step += 2) {
                {
                    const int s1 = step + 1;
                    const bool own = s1 < nk_self;
                    load_chunk(own ? a_self : a_agg, own ? s1 : s1 - nk_self, a1);
                }
                __builtin_amdgcn_sched_barrier(0);
                compute(step, a0);
                {
                    const int s2 = step + 2;
                    const float* nxt = (const float*)(h_src + (r_next >= 0 ? (int64_t)s_next * src_stride : 0)) + 16 * half;
                    // past the last step: step 0 of the next task's own half
                    const float* base = s2 < nk_self ? a_self : (s2 < nk ? a_agg : nxt);
                    const int c = s2 < nk_self ? s2 : (s2 < nk ? s2 - nk_self : 0);
                    load_chunk(base, c, a0);
                }
                __builtin_amdgcn_sched_barrier(0);
                compute(step + 1, a1);
            }
            // accumulator element i is row 8*(i/4) + 4*half + i%4 of the block, column l32 of its column block: the
            // destination rows of elements 4q .. 4q+3 are four consecutive entries of the list
            int32_t rr[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const i32x4 four = *(const i32x4*)(rowlist + tk * 32 + 8 * q + 4 * half);
#pragma unroll
                for (int u = 0; u < 4; ++u) rr[4 * q + u] = four[u];
            }
            // A block whose 32 rows are all in range and whose columns all exist (every block but the ragged last ones)
            // is stored without a condition per element: 32 branches would put every store in a basic block of its own.
            const bool whole = __all(r >= 0) && n0 + BNW <= d_out;
            if (whole && near_out) {
                // every byte offset into h_out fits 31 bits and rows and stride fit 24: one full-rate multiply per row,
                // shared by the column blocks, and the stores take the uniform base with a 32-bit offset
                const uint32_t col_off = (uint32_t)(n0 + l32) * 4u;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t row_off = __umul24((uint32_t)rr[i], (uint32_t)out_stride) + col_off;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        float v = (float)((double)big[nb][i] + (double)small[nb][i] + bv[nb]);
                        if (relu) v = fmaxf(v, 0.f);
                        *(float*)(h_out + (size_t)(row_off + (uint32_t)nb * 128u)) = v;
                    }
                }
            } else if (whole) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    char* out_col = h_out + (int64_t)(n0 + nb * 32 + l32) * 4;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float v = (float)((double)big[nb][i] + (double)small[nb][i] + bv[nb]);
                        if (relu) v = fmaxf(v, 0.f);
                        *(float*)(out_col + (int64_t)rr[i] * out_stride) = v;
                    }
                }
            } else {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int c = n0 + nb * 32 + l32;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float v = (float)((double)big[nb][i] + (double)small[nb][i] + bv[nb]);
                        if (relu) v = fmaxf(v, 0.f);
                        if (rr[i] >= 0 && c < d_out) *(float*)(h_out + (int64_t)rr[i] * out_stride + (int64_t)c * 4) = v;
                    }
                }
            }
            r = r_next;
            s = s_next;
            a_self = (const float*)(h_src + (r >= 0 ? (int64_t)s * src_stride : 0)) + 16 * half;
            a_agg = (const float*)(agg + (r >= 0 ? ((rb + stride) * 32 + l32) * agg_stride : 0)) + 16 * half;
        }
    }
}

// Few rows (fg_linear takes it up to 288 tasks: measured crossover with the bf16 x 3 panel kernel at 256 columns between
// 1024 and 1280 rows; fg_aggregate_linear up to 768):
// one workgroup per task, the K range split over its
// 8 wavefronts. A wavefront copies only its own rows of the W panel to LDS, fetches its A values in one round of
// loads, runs its one or two K chunks and leaves a 32 x 32 partial sum in fp64; the partial sums meet in LDS (in the
// space of the panel) and are added in wavefront order, so the result does not depend on timing. This removes the
// two costs that dominate a small layer in the panel kernel: a full pass over K by a single wavefront and the
// copy of a whole panel for a single task.
constexpr int SK_PART_BYTES = PL_WAVES * 16 * 64 * 8;  // partial sums: [wavefront][accumulator element][lane] doubles

// FUSE: the neighbour means are not read from `agg` but formed here from the block (fg_aggregate's arithmetic: fp64 sum
// in neighbour order, one division, one rounding to fp32), so a layer with few rows needs one launch instead of two.
template <bool FUSE>
__global__ __launch_bounds__(PL_THREADS, 2) void linear_f32_splitk_kernel(
    const char* __restrict__ h_src, int n_src, int64_t src_stride, const char* __restrict__ agg, int64_t agg_stride,
    const int32_t* __restrict__ rows, const int64_t* __restrict__ n_rows_dev, int64_t max_rows, int d_in, int d_out,
    const float* __restrict__ W, const float* __restrict__ bias, int relu, char* __restrict__ h_out, int n_out,
    int64_t out_stride, int n_panels, const int32_t* __restrict__ row_start, const int32_t* __restrict__ row_end,
    const int32_t* __restrict__ col, int64_t nnz, int n_block_rows, const int32_t* __restrict__ src_ids) {
    extern __shared__ __attribute__((aligned(16))) float panel[];  // [K][32], later the partial sums
    int64_t n_rows = n_rows_dev ? *n_rows_dev : max_rows;
    if (n_rows > max_rows) n_rows = max_rows;
    const int K = 2 * d_in;
    const int nk = K / KC, nk_self = d_in / KC;
    const int xcd = blockIdx.x & 7;
    const int j = blockIdx.x >> 3;
    const int n0 = (j % n_panels) * PL_BN;
    const int64_t rb = (int64_t)(j / n_panels) * 8 + xcd;  // the panels of a row block run on one XCD
    if (rb * 32 >= n_rows) return;                         // uniform over the workgroup, before any barrier
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    // The K chunks of this wavefront: chunk_of(0 .. cnt-1). Contiguous ranges, or with FUSE every eighth chunk, so that
    // each wavefront gets chunks of the self half and of the mean half (the means cost several loads per value).
    const int per = (nk + PL_WAVES - 1) / PL_WAVES;
    const int c0 = wave * per < nk ? wave * per : nk;
    const int c1 = c0 + per < nk ? c0 + per : nk;
    const int cnt = FUSE ? (nk > wave ? (nk - wave + PL_WAVES - 1) / PL_WAVES : 0) : c1 - c0;
    auto chunk_of = [&](int i) { return FUSE ? wave + i * PL_WAVES : c0 + i; };

    // destination / source row of this lane (-1: past the end or out of range; such a lane reads row 0)
    const int64_t g = rb * 32 + l32;
    int32_t r = -1, s_own = -1;
    if (g < n_rows) {
        r = rows ? rows[g] : (int32_t)g;
        if (r < 0 || r >= n_out) r = -1;
        s_own = own_row(src_ids, r, n_src);
        if (s_own < 0) r = -1;
    }
    const float* a_self = (const float*)(h_src + (r >= 0 ? (int64_t)s_own * src_stride : 0)) + 16 * half;
    const float* a_agg = (const float*)(agg + (r >= 0 ? g * agg_stride : 0)) + 16 * half;
    auto a_ptr = [&](int s) { return s < nk_self ? a_self + s * KC : a_agg + (s - nk_self) * KC; };
    // this lane's row of the block (FUSE): its sampled neighbours are col[e0 .. e1)
    int32_t e0 = 0, e1 = 0;
    if (FUSE && r >= 0 && r < n_block_rows) {
        e0 = row_start[r];
        e1 = row_end[r];
        if (e0 < 0 || e1 < e0 || (int64_t)e1 > nnz) e0 = e1 = 0;
    }
    // the 16 values of chunk s this lane feeds to the matrix instructions
    constexpr int NBF = 5;  // neighbours whose pieces are in flight together (the seed layer's fan-out)
    auto load_chunk = [&](int s, f32x4* a) {
        if (!FUSE || s < nk_self) {
            const float* p = a_ptr(s);
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] = *(const f32x4*)(p + 4 * q);
            return;
        }
        double acc[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.0;
        const int64_t off = ((int64_t)(s - nk_self) * KC + 16 * half) * 4;
        for (int e = e0; e < e1; e += NBF) {
            f32x4 v[NBF][4];
            bool ok[NBF];
            int32_t cc[NBF];
#pragma unroll
            for (int u = 0; u < NBF; ++u) cc[u] = col[e + u < e1 ? e + u : e0];  // all positions first, then all rows
#pragma unroll
            for (int u = 0; u < NBF; ++u) {
                const int32_t c = e + u < e1 ? cc[u] : -1;
                ok[u] = c >= 0 && c < n_src;
                const float* p = (const float*)(h_src + (ok[u] ? (int64_t)c * src_stride : 0) + off);
#pragma unroll
                for (int q = 0; q < 4; ++q) v[u][q] = *(const f32x4*)(p + 4 * q);
            }
#pragma unroll
            for (int u = 0; u < NBF; ++u)
                if (ok[u])
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] += (double)v[u][i >> 2][i & 3];
        }
        const double deg = (double)(e1 - e0);
#pragma unroll
        for (int i = 0; i < 16; ++i) a[i >> 2][i & 3] = deg > 0.0 ? (float)(acc[i] / deg) : 0.f;
    };

    // the first round of A loads goes out before anything else waits on memory
    f32x4 a0[4], a1[4];
    load_chunk(cnt > 0 ? chunk_of(0) : 0, a0);
    load_chunk(cnt > 1 ? chunk_of(1) : (cnt > 0 ? chunk_of(0) : 0), a1);
    // this wavefront's rows of the panel
    for (int q = lane; q < cnt * KC * 8; q += 64) {
        const int idx = q >> 3, c4 = (q & 7) * 4;
        const int k = chunk_of(idx / KC) * KC + idx % KC;
        const f32x4 v = *(const f32x4*)(W + (int64_t)k * d_out + (n0 + c4 < d_out ? n0 + c4 : 0));
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        *(f32x4*)(panel + k * PL_BN + c4) = n0 + c4 < d_out ? v : z;
    }
    double sum[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) sum[i] = 0.0;
    __syncthreads();
    const float* bcol = panel + 16 * half * PL_BN + l32;
    auto compute = [&](int s, const f32x4* a) {
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        const float* brow = bcol + s * KC * PL_BN;
#pragma unroll
        for (int q = 0; q < 16; ++q)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q >> 2][q & 3], brow[q * PL_BN], acc, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) sum[i] += (double)acc[i];
    };
    for (int i = 0; i < cnt; i += 2) {  // two chunks per round of loads (a chunk past the end re-reads chunk i)
        const bool two = i + 1 < cnt;
        if (i > 0) {
            load_chunk(chunk_of(i), a0);
            load_chunk(chunk_of(two ? i + 1 : i), a1);
        }
        compute(chunk_of(i), a0);
        if (two) compute(chunk_of(i + 1), a1);
    }
    __syncthreads();  // every wavefront is done with the panel: its space now takes the partial sums
    double* part = (double*)panel;
#pragma unroll
    for (int i = 0; i < 16; ++i) part[(wave * 16 + i) * 64 + lane] = sum[i];
    __syncthreads();
    const int c = n0 + l32;
    const double bv = (bias && c < d_out) ? (double)bias[c] : 0.0;
    // wavefront w finishes accumulator elements 2w and 2w+1: element i is row 8*(i/4) + 4*half + i%4 of the block
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int i = 2 * wave + e;
        double v = bv;
#pragma unroll
        for (int w = 0; w < PL_WAVES; ++w) v += part[(w * 16 + i) * 64 + lane];
        const int m = 8 * (i >> 2) + 4 * half + (i & 3);
        const int32_t rr = __shfl(r, m, 64);  // lane m (< 32) holds the destination row of block row m; all lanes active
        if (rr < 0 || c >= d_out) continue;
        float o = (float)v;
        if (relu) o = o > 0.f ? o : 0.f;
        *(float*)(h_out + (int64_t)rr * out_stride + (int64_t)c * 4) = o;
    }
}

}  // namespace

fg_status_t fg_launch_linear_bf16(const void* h_src, int32_t n_src, int64_t src_stride, fg_dtype_t in_dtype,
                                  const void* agg, int64_t agg_stride, const int32_t* rows_dev,
                                  const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in, int32_t d_out, const void* W,
                                  const float* bias, int32_t relu, void* h_out, int32_t n_out, int64_t out_stride,
                                  fg_dtype_t out_dtype, hipStream_t st, bool w_nk, const int64_t* k_limit_dev = nullptr,
                                  const int32_t* src_ids_dev = nullptr);

// fg_linear (src_ids_dev == NULL: the own features of position r are row r of h_src) and fg_linear_ids (row src_ids_dev[r])
static fg_status_t linear_launch(const char* who, const void* h_src, int32_t n_src, int64_t src_stride, fg_dtype_t in_dtype,
                                 const int32_t* src_ids_dev, const void* agg, int64_t agg_stride, const int32_t* rows_dev,
                                 const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in, int32_t d_out, const void* W,
                                 fg_dtype_t w_dtype, const float* bias, int32_t relu, void* h_out, int32_t n_out,
                                 int64_t out_stride, fg_dtype_t out_dtype, void* stream) {
    if (max_rows < 0 || n_src < 0 || n_out < 0 || d_in <= 0 || d_out <= 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: bad size (max_rows %lld, n_src %d, n_out %d, d_in %d, d_out %d)", who,
                (long long)max_rows, n_src, n_out, d_in, d_out);
    if (!fg_dtype_size(in_dtype) || !fg_dtype_size(w_dtype) || !fg_dtype_size(out_dtype))
        FG_FAIL(FG_ERR_DTYPE, "%s: unknown element type", who);
    if (max_rows > 0 && (!h_src || !agg || !W || !h_out)) FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    hipStream_t st = (hipStream_t)stream;
    if (w_dtype == FG_F32) {
        if (in_dtype != FG_F32 || out_dtype != FG_F32)
            FG_FAIL(FG_ERR_DTYPE, "%s: fp32 weights need fp32 inputs and outputs", who);
        if (d_in % 4 || d_out % 4) FG_FAIL(FG_ERR_SHAPE, "%s: d_in = %d and d_out = %d must be multiples of 4", who, d_in, d_out);
        if (src_stride < (int64_t)d_in * 4 || agg_stride < (int64_t)d_in * 4 || out_stride < (int64_t)d_out * 4)
            FG_FAIL(FG_ERR_SHAPE, "%s: a row stride is smaller than its row", who);
        if (((uintptr_t)h_src | (uintptr_t)agg | (uintptr_t)W | (uintptr_t)src_stride | (uintptr_t)agg_stride) & 15)
            FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_src, agg, W and the input strides must be 16-byte aligned", who);
        if (((uintptr_t)h_out | (uintptr_t)out_stride | (uintptr_t)bias) & 3)
            FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_out, its stride and bias must be 4-byte aligned", who);
        fg_clear_error();
        if (max_rows == 0) return FG_OK;
        const int64_t forced = fg_tuning(FG_TUNE_LINEAR_TILE);
        const size_t panel_bytes = (size_t)2 * d_in * PL_BN * sizeof(float);
        if (n_src == 0 || n_out == 0) return FG_OK;  // no row can be in range
        const int64_t n_tasks = fg_ceil_div(max_rows, 32) * fg_ceil_div(d_out, PL_BN);
        if (d_in % KC == 0 && panel_bytes <= 64 * 1024 && (forced == 8 || (forced == 0 && n_tasks <= 288))) {
            const int n_panels = (int)fg_ceil_div(d_out, PL_BN);
            const size_t lds = panel_bytes > (size_t)SK_PART_BYTES ? panel_bytes : (size_t)SK_PART_BYTES;
            const unsigned grid = (unsigned)(fg_ceil_div(fg_ceil_div(max_rows, 32), 8) * 8 * n_panels);
            hipLaunchKernelGGL(linear_f32_splitk_kernel<false>, dim3(grid), dim3(PL_THREADS), lds, st, (const char*)h_src, n_src,
                               src_stride, (const char*)agg, agg_stride, rows_dev, n_rows_dev, max_rows, d_in, d_out,
                               (const float*)W, bias, relu, (char*)h_out, n_out, out_stride, n_panels, nullptr, nullptr, nullptr,
                               (int64_t)0, 0, src_ids_dev);
            FG_LAUNCH_CHECK("linear_f32_splitk_kernel");
            return FG_OK;
        }
        // bf16 x 3 panel kernel: two 32-column blocks per wavefront if the split panel fits in LDS, else one. A d_in that is
        // not a multiple of 32 is walked as the next multiple (zero weights, zero pieces: the RAGGED variant).
        const int d_pad = (int)(fg_ceil_div(d_in, KC) * KC);
        const bool ragged = d_pad != d_in;
        const size_t x3_bytes = (size_t)2 * d_pad * 192;
        const size_t x3_lists = (size_t)X3_LIST_BYTES * (src_ids_dev ? 2 : 1);
        if (x3_bytes + x3_lists <= 160 * 1024 && x3_bytes <= 144 * 1024 && (forced == 0 || forced == 301 || forced == 302)) {
            const int nb = (forced != 301 && 2 * x3_bytes <= 144 * 1024) ? 2 : 1;
            const size_t lds = x3_bytes * nb + x3_lists;          // fragments of the panel, then the wavefronts' row lists
            const int n_panels = (int)fg_ceil_div(d_out, PL_BN * nb);
            int q = 256 / (8 * n_panels);  // register use allows one workgroup per compute unit
            if (q < 1) q = 1;
            const int64_t blocks32 = fg_ceil_div(max_rows, 32);
            while (q > 1 && (int64_t)8 * (q - 1) >= blocks32) --q;
            const int n_groups = 8 * q;
            // output offsets in 32 bits: every byte of h_out below 2^31, rows and stride below 2^24
            const int near_out = ((int64_t)n_out * out_stride < (1ll << 31) && n_out < (1 << 24) && out_stride < (1 << 24)) ? 1 : 0;
#define FG_X3(NBV, RAG)                                                                                                        \
    hipLaunchKernelGGL((linear_f32x3_panel_kernel<NBV, RAG>), dim3((unsigned)(n_groups * n_panels)), dim3(PL_THREADS), lds, st,  \
                       (const char*)h_src, n_src, src_stride, (const char*)agg, agg_stride, rows_dev, n_rows_dev, max_rows, d_in, \
                       d_out, (const float*)W, bias, relu, (char*)h_out, n_out, out_stride, n_panels, n_groups, near_out, src_ids_dev)
            if (nb == 2) {
                if (ragged) FG_X3(2, true); else FG_X3(2, false);
            } else {
                if (ragged) FG_X3(1, true); else FG_X3(1, false);
            }
#undef FG_X3
            FG_LAUNCH_CHECK("linear_f32x3_panel_kernel");
            return FG_OK;
        }
        if (d_in % KC == 0 && panel_bytes <= 64 * 1024 && (forced == 0 || forced == 32)) {  // fp32 matrix instructions
            const int n_panels = (int)fg_ceil_div(d_out, PL_BN);
            // two workgroups (of eight wavefronts) per compute unit; 8 * q groups of workgroups, each group holding all panels
            int q = (2 * 256) / (8 * n_panels);
            if (q < 1) q = 1;
            const int64_t blocks32 = fg_ceil_div(max_rows, 32);
            while (q > 1 && (int64_t)8 * (q - 1) >= blocks32) --q;  // no more groups than row blocks
            const int n_groups = 8 * q;
            hipLaunchKernelGGL(linear_f32_panel_kernel, dim3((unsigned)(n_groups * n_panels)), dim3(PL_THREADS), panel_bytes, st,
                               (const char*)h_src, n_src, src_stride, (const char*)agg, agg_stride, rows_dev, n_rows_dev,
                               max_rows, d_in, d_out, (const float*)W, bias, relu, (char*)h_out, n_out, out_stride, n_panels,
                               n_groups, src_ids_dev);
            FG_LAUNCH_CHECK("linear_f32_panel_kernel");
            return FG_OK;
        }
        const int ny = (int)fg_ceil_div(d_out, BN);
        // 64-row tiles (four workgroups per compute unit) measured faster than 128-row tiles at every layer size
        const bool big = forced >= 128;
        const int64_t m_tiles = fg_ceil_div(max_rows, big ? 128 : 64);
        const unsigned grid = (unsigned)(fg_ceil_div(m_tiles, 8) * 8 * ny);
        if (big)
            hipLaunchKernelGGL((linear_f32_kernel<4, 32>), dim3(grid), dim3(LIN_THREADS), 0, st, (const char*)h_src, n_src, src_stride,
                               (const char*)agg, agg_stride, rows_dev, n_rows_dev, max_rows, d_in, d_out, (const float*)W,
                               bias, relu, (char*)h_out, n_out, out_stride, ny, src_ids_dev);
        else
            hipLaunchKernelGGL((linear_f32_kernel<2, 32>), dim3(grid), dim3(LIN_THREADS), 0, st, (const char*)h_src, n_src, src_stride,
                               (const char*)agg, agg_stride, rows_dev, n_rows_dev, max_rows, d_in, d_out, (const float*)W,
                               bias, relu, (char*)h_out, n_out, out_stride, ny, src_ids_dev);
        FG_LAUNCH_CHECK("linear_f32_kernel");
        return FG_OK;
    }
    if (w_dtype == FG_BF16)
        return fg_launch_linear_bf16(h_src, n_src, src_stride, in_dtype, agg, agg_stride, rows_dev, n_rows_dev, max_rows,
                                     d_in, d_out, W, bias, relu, h_out, n_out, out_stride, out_dtype, st, false, nullptr, src_ids_dev);
    FG_FAIL(FG_ERR_DTYPE, "%s: weights must be F32 or BF16", who);
}

extern "C" fg_status_t fg_linear(const void* h_src, int32_t n_src, int64_t src_stride, fg_dtype_t in_dtype,
                                 const void* agg, int64_t agg_stride, const int32_t* rows_dev,
                                 const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in, int32_t d_out, const void* W,
                                 fg_dtype_t w_dtype, const float* bias, int32_t relu, void* h_out, int32_t n_out,
                                 int64_t out_stride, fg_dtype_t out_dtype, void* stream) {
    return linear_launch("fg_linear", h_src, n_src, src_stride, in_dtype, nullptr, agg, agg_stride, rows_dev, n_rows_dev, max_rows,
                         d_in, d_out, W, w_dtype, bias, relu, h_out, n_out, out_stride, out_dtype, stream);
}

// fg_linear with the own features read straight from a table: row src_ids_dev[r] of `table` for output position r
extern "C" fg_status_t fg_linear_ids(const void* table, int32_t table_rows, int64_t src_stride, fg_dtype_t in_dtype,
                                     const int32_t* src_ids_dev, const void* agg, int64_t agg_stride, const int32_t* rows_dev,
                                     const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in, int32_t d_out, const void* W,
                                     fg_dtype_t w_dtype, const float* bias, int32_t relu, void* h_out, int32_t n_out,
                                     int64_t out_stride, fg_dtype_t out_dtype, void* stream) {
    if (max_rows > 0 && n_out > 0 && !src_ids_dev) FG_FAIL(FG_ERR_INVALID_ARG, "fg_linear_ids: src_ids_dev is NULL");
    return linear_launch("fg_linear_ids", table, table_rows, src_stride, in_dtype, src_ids_dev, agg, agg_stride, rows_dev, n_rows_dev,
                         max_rows, d_in, d_out, W, w_dtype, bias, relu, h_out, n_out, out_stride, out_dtype, stream);
}

// fg_linear with the bf16 weights given transposed ([d_out x 2*d_in], one output column's weights contiguous): the layout
// the matrix-core kernel reads 16 bytes at a time, with no reshuffling on the way into LDS.
extern "C" fg_status_t fg_linear_wt(const void* h_src, int32_t n_src, int64_t src_stride, fg_dtype_t in_dtype, const void* agg,
                                    int64_t agg_stride, const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                                    int32_t d_in, int32_t d_out, const void* Wt, fg_dtype_t w_dtype, const float* bias, int32_t relu,
                                    void* h_out, int32_t n_out, int64_t out_stride, fg_dtype_t out_dtype, void* stream) {
    if (max_rows < 0 || n_src < 0 || n_out < 0 || d_in <= 0 || d_out <= 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "fg_linear_wt: bad size (max_rows %lld, n_src %d, n_out %d, d_in %d, d_out %d)",
                (long long)max_rows, n_src, n_out, d_in, d_out);
    if (w_dtype != FG_BF16) FG_FAIL(FG_ERR_DTYPE, "fg_linear_wt: transposed weights are taken in bf16 only");
    if (max_rows > 0 && (!h_src || !agg || !Wt || !h_out)) FG_FAIL(FG_ERR_INVALID_ARG, "fg_linear_wt: NULL pointer");
    return fg_launch_linear_bf16(h_src, n_src, src_stride, in_dtype, agg, agg_stride, rows_dev, n_rows_dev, max_rows, d_in, d_out,
                                 Wt, bias, relu, h_out, n_out, out_stride, out_dtype, (hipStream_t)stream, true);
}


// fg_aggregate followed by fg_linear for one fp32 layer. A layer with few rows (the seed layer) runs as one launch that
// forms the neighbour means while it loads its operands; any other shape runs the two calls, with agg_ws_dev between them.
extern "C" fg_status_t fg_aggregate_linear(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                                           int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                           int64_t max_rows, const float* h_src, int32_t n_src, int64_t src_stride, int32_t d_in,
                                           int32_t d_out, const float* W, const float* bias, int32_t relu, float* agg_ws_dev,
                                           int64_t agg_stride, float* h_out, int32_t n_out, int64_t out_stride, void* stream) {
    const char* who = "fg_aggregate_linear";
    if (max_rows < 0 || n_block_rows < 0 || n_src < 0 || n_out < 0 || nnz < 0 || d_in <= 0 || d_out <= 0)
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: bad size", who);
    if (max_rows > 0 && (!row_start_dev || !row_end_dev || !h_src || !W || !h_out || (nnz > 0 && !col_dev)))
        FG_FAIL(FG_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (d_in % 4 || d_out % 4) FG_FAIL(FG_ERR_SHAPE, "%s: d_in = %d and d_out = %d must be multiples of 4", who, d_in, d_out);
    if (src_stride < (int64_t)d_in * 4 || out_stride < (int64_t)d_out * 4) FG_FAIL(FG_ERR_SHAPE, "%s: a row stride is smaller than its row", who);
    if (((uintptr_t)h_src | (uintptr_t)W | (uintptr_t)src_stride) & 15) FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_src, W and src_stride must be 16-byte aligned", who);
    if (((uintptr_t)h_out | (uintptr_t)out_stride | (uintptr_t)bias) & 3) FG_FAIL(FG_ERR_INVALID_ARG, "%s: h_out, its stride and bias must be 4-byte aligned", who);
    const size_t panel_bytes = (size_t)2 * d_in * PL_BN * sizeof(float);
    const int64_t n_tasks = fg_ceil_div(max_rows, 32) * fg_ceil_div(d_out, PL_BN);
    const int64_t forced = fg_tuning(FG_TUNE_LINEAR_TILE);
    if (d_in % KC == 0 && panel_bytes <= 64 * 1024 && n_tasks <= 768 && (forced == 0 || forced == 8)) {
        fg_clear_error();
        if (max_rows == 0 || n_src == 0 || n_out == 0) return FG_OK;
        const int n_panels = (int)fg_ceil_div(d_out, PL_BN);
        const size_t lds = panel_bytes > (size_t)SK_PART_BYTES ? panel_bytes : (size_t)SK_PART_BYTES;
        const unsigned grid = (unsigned)(fg_ceil_div(fg_ceil_div(max_rows, 32), 8) * 8 * n_panels);
        hipLaunchKernelGGL(linear_f32_splitk_kernel<true>, dim3(grid), dim3(PL_THREADS), lds, (hipStream_t)stream, (const char*)h_src,
                           n_src, src_stride, (const char*)h_src, src_stride, rows_dev, n_rows_dev, max_rows, d_in, d_out, W, bias, relu,
                           (char*)h_out, n_out, out_stride, n_panels, row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, nullptr);
        FG_LAUNCH_CHECK("linear_f32_splitk_kernel (fused aggregation)");
        return FG_OK;
    }
    if (max_rows > 0 && !agg_ws_dev) FG_FAIL(FG_ERR_INVALID_ARG, "%s: this shape runs as two launches and needs agg_ws_dev", who);
    fg_status_t rc = fg_aggregate(row_start_dev, row_end_dev, col_dev, nnz, n_block_rows, rows_dev, n_rows_dev, max_rows, h_src, n_src,
                                  src_stride, d_in, FG_F32, agg_ws_dev, agg_stride, FG_F32, stream);
    if (rc != FG_OK) return rc;
    return fg_linear(h_src, n_src, src_stride, FG_F32, agg_ws_dev, agg_stride, rows_dev, n_rows_dev, max_rows, d_in, d_out, W, FG_F32,
                     bias, relu, h_out, n_out, out_stride, FG_F32, stream);
}
