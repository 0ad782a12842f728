/* A caller of the library in plain C: no Python, no torch, only the HIP runtime's C API for device memory. It gathers rows of
 * a table by index (fg_gather), aggregates a small block (fg_aggregate), creates, clears and destroys a cache, and then runs
 * two iterations of a one-layer cached path by hand (fg_lookup_prune, fg_linear with identity panels, fg_cache_update, the
 * lookup of the next iteration, the fetch of the cached rows), checking every result on the host against values worked out
 * in the comments. Exit status 0 and "ok" on success. Built by __graft_entry__.build() with gcc. */
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
    {
        /* Two iterations over one cached layer: nodes 10, 20, 30, 40 at positions 0..3, the block above over 5 source positions
         * (its last column, 999, is out of range and ignored). Iteration 0: the cache is empty, every row is normal.
         * Norms 1, 2, 3, 4 with p_grad = 0.5: k = 2, tau = 3, so nodes 10 and 20 are admitted into slots 0 and 1.
         * Iteration 1: positions 0 and 1 hit, their rows are cut (end = start); rows 2 and 3 stay and keep positions
         * 2, 0, 2, 4 and 3 of the layer below alive: liveness 1 0 1 1 1. */
        enum { NS = 5 };
        const int32_t ids[N] = {10, 20, 30, 40};
        const float gnorm[N] = {1.f, 2.f, 3.f, 4.f};
        static float W[2 * DIM][DIM], hout[N][DIM], fetched[2][DIM];
        int32_t *d_ids, *d_hp, *d_hs, *d_np;
        uint8_t *d_hit, *d_live_src;
        int64_t *d_counts, *d_stats;
        float *d_gn, *d_W, *d_hout, *d_fetched;
        void* d_ws;
        size_t ws_bytes = fg_workspace_bytes(FG_WS_LOOKUP_PRUNE, N, 0);
        if (fg_workspace_bytes(FG_WS_CACHE_UPDATE, N, 0) > ws_bytes) ws_bytes = fg_workspace_bytes(FG_WS_CACHE_UPDATE, N, 0);
        if (!ws_bytes) return 9;
        CHECK_HIP(hipMalloc((void**)&d_ids, sizeof ids));
        CHECK_HIP(hipMalloc((void**)&d_hp, sizeof ids));
        CHECK_HIP(hipMalloc((void**)&d_hs, sizeof ids));
        CHECK_HIP(hipMalloc((void**)&d_np, sizeof ids));
        CHECK_HIP(hipMalloc((void**)&d_hit, N));
        CHECK_HIP(hipMalloc((void**)&d_live_src, NS));
        CHECK_HIP(hipMalloc((void**)&d_counts, 3 * sizeof(int64_t)));
        CHECK_HIP(hipMalloc((void**)&d_stats, 4 * sizeof(int64_t)));
        CHECK_HIP(hipMalloc((void**)&d_gn, sizeof gnorm));
        CHECK_HIP(hipMalloc((void**)&d_W, sizeof W));
        CHECK_HIP(hipMalloc((void**)&d_hout, sizeof hout));
        CHECK_HIP(hipMalloc((void**)&d_fetched, sizeof fetched));
        CHECK_HIP(hipMalloc(&d_ws, ws_bytes));
        CHECK_HIP(hipMemcpy(d_ids, ids, sizeof ids, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemcpy(d_gn, gnorm, sizeof gnorm, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemset(d_stats, 0, 4 * sizeof(int64_t)));
        int64_t counts[3], stats[4];
        int32_t pos[N], slot[N], end_now[N];
        uint8_t hit[N], live_src[NS];

        /* iteration 0: lookup, prune, V_normal */
        CHECK_FG(fg_lookup_prune(cache, 1, 0, d_ids, N, NULL, d_start, d_end, d_col, NNZ, NS, d_live_src, d_hit, d_hp, d_hs, d_np, NULL,
                                 d_counts, d_ws, ws_bytes, NULL));
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(counts, d_counts, sizeof counts, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(pos, d_np, sizeof pos, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(live_src, d_live_src, sizeof live_src, hipMemcpyDeviceToHost));
        if (counts[0] != 4 || counts[1] != 0 || counts[2] != 4 || pos[0] != 0 || pos[1] != 1 || pos[2] != 2 || pos[3] != 3) return 10;
        for (int j = 0; j < NS; ++j)
            if (live_src[j] != 1) return 11;
        /* dense update with W = [I; 0]: the rows' own previous embeddings (table rows 0..3), bit for bit; with [0; I]: the means */
        for (int half = 0; half < 2; ++half) {
            memset(W, 0, sizeof W);
            for (int c = 0; c < DIM; ++c) W[half * DIM + c][c] = 1.0f;
            CHECK_HIP(hipMemcpy(d_W, W, sizeof W, hipMemcpyHostToDevice));
            CHECK_FG(fg_linear(d_table, ROWS, DIM * 4, FG_F32, d_agg, DIM * 4, d_np, d_counts + 2, N, DIM, DIM, d_W, FG_F32, NULL, 0,
                               d_hout, N, DIM * 4, FG_F32, NULL));
            CHECK_HIP(hipDeviceSynchronize());
            CHECK_HIP(hipMemcpy(hout, d_hout, sizeof hout, hipMemcpyDeviceToHost));
            for (int k = 0; k < N; ++k)
                if (memcmp(hout[k], half == 0 ? table[k] : agg[k], sizeof hout[k]) != 0) {
                    fprintf(stderr, "fg_linear with an identity panel (%d): row %d differs\n", half, k);
                    return 12;
                }
        }
        /* update: d_hout holds the means; nodes 10 and 20 are admitted with them */
        CHECK_FG(fg_cache_update(cache, 1, 0, d_ids, N, NULL, d_hit, d_gn, 0.5f, d_hout, DIM * 4, d_stats, d_ws, ws_bytes, NULL));
        /* iteration 1 */
        CHECK_FG(fg_lookup_prune(cache, 1, 1, d_ids, N, NULL, d_start, d_end, d_col, NNZ, NS, d_live_src, d_hit, d_hp, d_hs, d_np, NULL,
                                 d_counts, d_ws, ws_bytes, NULL));
        CHECK_FG(fg_gather(fg_cache_table(cache, 1), 128, DIM * 4, DIM * 4, d_hs, NULL, d_counts + 1, 2, d_fetched, 2, DIM * 4,
                           FG_TABLE_HBM_REUSED, NULL));
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(stats, d_stats, sizeof stats, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(counts, d_counts, sizeof counts, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(pos, d_hp, sizeof pos, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(slot, d_hs, sizeof slot, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(hit, d_hit, sizeof hit, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(end_now, d_end, sizeof end_now, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(live_src, d_live_src, sizeof live_src, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(fetched, d_fetched, sizeof fetched, hipMemcpyDeviceToHost));
        if (stats[0] != 2 || stats[1] != 0 || stats[2] != 0 || stats[3] != 0) return 13;
        if (counts[0] != 4 || counts[1] != 2 || counts[2] != 2) return 14;
        if (pos[0] != 0 || pos[1] != 1 || slot[0] != 0 || slot[1] != 1 || hit[0] != 1 || hit[1] != 1 || hit[2] != 0 || hit[3] != 0) return 15;
        if (end_now[0] != row_start[0] || end_now[1] != row_start[1] || end_now[2] != row_end[2] || end_now[3] != row_end[3]) return 16;
        if (live_src[0] != 1 || live_src[1] != 0 || live_src[2] != 1 || live_src[3] != 1 || live_src[4] != 1) return 17;
        if (memcmp(fetched[0], agg[0], sizeof fetched[0]) != 0 || memcmp(fetched[1], agg[1], sizeof fetched[1]) != 0) return 18;
        hipFree(d_ids); hipFree(d_hp); hipFree(d_hs); hipFree(d_np); hipFree(d_hit); hipFree(d_live_src); hipFree(d_counts);
        hipFree(d_stats); hipFree(d_gn); hipFree(d_W); hipFree(d_hout); hipFree(d_fetched); hipFree(d_ws);
    }
    CHECK_FG(fg_cache_destroy(cache));
    hipFree(d_table); hipFree(d_got); hipFree(d_agg); hipFree(d_index); hipFree(d_start); hipFree(d_end); hipFree(d_col);
    printf("ok\n");
    return 0;
}
