/* A caller of the library in plain C: no Python, no torch, only the HIP runtime's C API for device memory. It gathers rows of
 * a table by index (fg_gather), aggregates a small block (fg_aggregate) and creates, clears and destroys a cache, and checks
 * the results on the host. Exit status 0 and "ok" on success. Built by __graft_entry__.build() with gcc. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "freshgnn.h"

#define CHECK_HIP(x)                                                      \
    do {                                                                  \
        hipError_t e_ = (x);                                              \
        if (e_ != hipSuccess) {                                           \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));      \
            return 2;                                                     \
        }                                                                 \
    } while (0)
#define CHECK_FG(x)                                                       \
    do {                                                                  \
        if ((x) != FG_OK) {                                               \
            fprintf(stderr, "%s: %s\n", #x, fg_last_error());             \
            return 3;                                                     \
        }                                                                 \
    } while (0)

int main(void) {
    enum { ROWS = 1000, DIM = 64, PICK = 300, N = 4, NNZ = 6 };
    static float table[ROWS][DIM], got[PICK][DIM], agg[N][DIM];
    int32_t index[PICK], row_start[N] = {0, 2, 2, 5}, row_end[N] = {2, 2, 5, 6}, col[NNZ] = {1, 3, 0, 2, 4, 999};
    for (int r = 0; r < ROWS; ++r)
        for (int c = 0; c < DIM; ++c) table[r][c] = (float)(r * 131 % 977) + 0.25f * (float)c;
    for (int k = 0; k < PICK; ++k) index[k] = (k * 37 + 11) % ROWS;

    float *d_table, *d_got, *d_agg;
    int32_t *d_index, *d_start, *d_end, *d_col;
    CHECK_HIP(hipMalloc((void**)&d_table, sizeof table));
    CHECK_HIP(hipMalloc((void**)&d_got, sizeof got));
    CHECK_HIP(hipMalloc((void**)&d_agg, sizeof agg));
    CHECK_HIP(hipMalloc((void**)&d_index, sizeof index));
    CHECK_HIP(hipMalloc((void**)&d_start, sizeof row_start));
    CHECK_HIP(hipMalloc((void**)&d_end, sizeof row_end));
    CHECK_HIP(hipMalloc((void**)&d_col, sizeof col));
    CHECK_HIP(hipMemcpy(d_table, table, sizeof table, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_index, index, sizeof index, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_start, row_start, sizeof row_start, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_end, row_end, sizeof row_end, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_col, col, sizeof col, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(d_got, 0, sizeof got));
    CHECK_HIP(hipMemset(d_agg, 0xFF, sizeof agg));

    if (fg_version() < 200) return 4;
    /* dst[k] = table[index[k]] */
    CHECK_FG(fg_gather(d_table, ROWS, DIM * 4, DIM * 4, d_index, NULL, NULL, PICK, d_got, PICK, DIM * 4, FG_TABLE_HBM_STREAMED, NULL));
    /* agg[k] = mean of the neighbour rows of row k (rows 0..3 of the block, all of them listed: rows_dev NULL) */
    CHECK_FG(fg_aggregate(d_start, d_end, d_col, NNZ, N, NULL, NULL, N, d_table, ROWS, DIM * 4, DIM, FG_F32, d_agg, DIM * 4, FG_F32, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(got, d_got, sizeof got, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(agg, d_agg, sizeof agg, hipMemcpyDeviceToHost));
    for (int k = 0; k < PICK; ++k)
        if (memcmp(got[k], table[index[k]], sizeof got[k]) != 0) {
            fprintf(stderr, "gathered row %d differs\n", k);
            return 5;
        }
    for (int k = 0; k < N; ++k) {
        const int deg = row_end[k] - row_start[k];
        for (int c = 0; c < DIM; ++c) {
            double want = 0.0;
            for (int e = row_start[k]; e < row_end[k]; ++e) want += table[col[e]][c];
            want = deg ? want / deg : 0.0;
            const double err = (double)agg[k][c] - want;
            if (err > 1e-3 || err < -1e-3) {
                fprintf(stderr, "mean of row %d, column %d: %g instead of %g\n", k, c, (double)agg[k][c], want);
                return 6;
            }
        }
    }
    /* an argument the library must refuse on the host, with a message */
    if (fg_gather(d_table, ROWS, DIM * 4, DIM * 4 + 1, d_index, NULL, NULL, PICK, d_got, PICK, DIM * 4, 0, NULL) == FG_OK || !fg_last_error()[0])
        return 7;
    fg_cache_t* cache = NULL;
    const int64_t capacity[1] = {128};
    const int32_t dim[1] = {DIM};
    CHECK_FG(fg_cache_create(&cache, ROWS, 1, capacity, dim, FG_F32, 5, NULL));
    if (!cache || !fg_cache_table(cache, 1)) return 8;
    CHECK_FG(fg_cache_clear(cache, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_FG(fg_cache_destroy(cache));
    hipFree(d_table); hipFree(d_got); hipFree(d_agg); hipFree(d_index); hipFree(d_start); hipFree(d_end); hipFree(d_col);
    printf("ok\n");
    return 0;
}
