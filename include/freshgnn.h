/*
 * freshgnn.h - C ABI of the MI355X (gfx950) hot path of mini-batch GNN training with a
 * selective historical-embedding cache (Algorithm 1 of the paper).
 *
 * One training iteration calls, in this order:
 *   top-down   fg_lookup_prune  for layers L, L-1, ..., 1, 0   (cache lookup, pruning, V_normal)
 *   loader     fg_gather        raw features of the surviving input nodes
 *   bottom-up  for l = 1..L:    fg_gather (cached rows of V_cache; or fg_cache_fetch_all once for all layers),
 *                               fg_aggregate, fg_linear
 *   update     fg_cache_update  for l = 1..L-1   (or fg_cache_update_all once)
 * With raw features sharing the cache's buffer (fg_cache_create_bidirectional, fg_cache_fill_features) the loader is
 * fg_gather_features / fg_gather_aggregate_features.
 *
 * Conventions
 *   - Every pointer named *_dev or documented "device" is device memory owned by the caller
 *     (a pointer to host memory mapped into the device address space works wherever a table
 *     is only read; it is named where that is intended). "host" pointers are ordinary host memory.
 *   - All calls are asynchronous on the caller's stream (a hipStream_t passed as void*), never
 *     synchronise the device and never copy a count back to the host: element counts that are
 *     only known on the device are read from device memory by the kernels, and the host passes
 *     an upper bound (max_*) that sizes the launch.
 *   - Node ids, positions and slot indices are int32; byte strides are int64; counts on the
 *     device are int64.
 *   - A mini-batch layer l holds n_l distinct node ids by position. Block l (l >= 1) connects
 *     layer l-1 to layer l in the two-row-array format of Section 5: the sampled neighbours of
 *     row j are col[row_start[j] .. row_end[j]), each a position in layer l-1, and layer l-1
 *     begins with the nodes of layer l in the same order (row j's own previous embedding is at
 *     position j).
 *   - Return value: FG_OK or an error code; fg_last_error() gives the message for the calling
 *     thread. Arguments are validated on the host before anything is launched; a call that
 *     returns an error has launched nothing. Indices read from device memory are range-checked
 *     inside the kernels: an out-of-range entry is skipped, never dereferenced.
 *   - Calls on one cache must be ordered by the caller (same stream, or events); the library
 *     keeps no locks.
 */
#ifndef FRESHGNN_H
#define FRESHGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t fg_status_t;
enum {
    FG_OK = 0,
    FG_ERR_INVALID_ARG = 1, /* NULL where a pointer is required, negative size, bad enum, bad alignment */
    FG_ERR_SHAPE = 2,       /* sizes that do not fit together (layer index, dim, strides, workspace too small) */
    FG_ERR_DTYPE = 3,       /* element type not supported by this call */
    FG_ERR_STATE = 4,       /* call not valid in the cache's current state (e.g. iteration going backwards) */
    FG_ERR_OOM = 5,         /* device allocation failed */
    FG_ERR_HIP = 6          /* the HIP runtime reported an error (message in fg_last_error) */
};

typedef enum { FG_F32 = 0, FG_F16 = 1, FG_BF16 = 2 } fg_dtype_t;

typedef struct fg_cache fg_cache_t; /* opaque: the historical embedding caches C^(1..L-1) of one model */

/* Message of the last error on this thread ("" if none). The pointer stays valid until the next failing call. */
const char* fg_last_error(void);
/* Library version, major * 10000 + minor * 100 + patch. */
int32_t fg_version(void);

/*
 * Historical embedding cache (Section 4.2, embedding side): per cached layer a node-id mapping
 * array of length num_nodes (entry = slot or -1), a slot table [capacity x dim] of `dtype`, and a
 * ring header; per slot also the owning node and the iteration that admitted it.
 * A cached embedding admitted by the update of iteration a is usable by the lookups of
 * iterations a+1 .. a+t_stale (Section 4.1.2); t_stale = 0 therefore disables the cache.
 *
 * n_layers: number of cached layers; layer indices 1..n_layers are valid in the calls below
 * (for an L-layer model pass L-1). capacity[k], dim[k]: slots and row width of layer k+1 (host arrays).
 * The library allocates (hipMalloc) and owns all cache memory:
 *   num_nodes*4 + capacity*(dim*sizeof(dtype) + 8) bytes per layer; the slot tables of all layers lie in one buffer.
 * The initialisation is queued on `stream`. *out is NULL on error.
 */
fg_status_t fg_cache_create(fg_cache_t** out, int64_t num_nodes, int32_t n_layers, const int64_t* capacity,
                            const int32_t* dim, fg_dtype_t dtype, int32_t t_stale, void* stream);

/*
 * The bidirectional cache of Section 4.2: the same historical embedding cache, created inside a buffer of
 * `buffer_bytes` bytes (a multiple of 256, at least the rings' size) that raw features share.
 *   Embedding side: the slot table ("ring") of layer 1 starts at byte 0, every further layer's at the next
 *   multiple of 256 after the previous ring; slot s of a ring occupies [base + s*row, base + (s+1)*row).
 *   Feature side: fg_cache_fill_features places raw feature rows from the right end of the buffer.
 *   Junction: the two sides may overlap. A feature row is lost as soon as an embedding has been written over any
 *   of its bytes and not earlier; a ring writes its slots in increasing order until it first wraps, so what ring l
 *   has written is [base_l, base_l + used_l*row_l), used_l = number of distinct slots written since create/clear.
 * At most 8 cached layers. fg_cache_create is this call with a buffer that just holds the rings.
 */
fg_status_t fg_cache_create_bidirectional(fg_cache_t** out, int64_t num_nodes, int32_t n_layers, const int64_t* capacity,
                                          const int32_t* dim, fg_dtype_t dtype, int32_t t_stale, int64_t buffer_bytes,
                                          void* stream);
/*
 * Populates the feature side before training (Section 4.2): the raw feature row of hot_ids_dev[r] (device int32,
 * distinct node ids in decreasing order of estimated saved memory access; r = 0 is the most valuable) is copied from
 * `table` (device, or host memory mapped into the device address space; row v at table + v*src_stride) to the bytes
 * [buffer_bytes - (r+1)*row_bytes, buffer_bytes - r*row_bytes) of the buffer, so the least valuable rows are the
 * first an advancing ring overwrites. An id outside [0, min(num_nodes, table_rows)) leaves its rank unused.
 * Only valid while the embedding side is empty (after create or fg_cache_clear; FG_ERR_STATE otherwise);
 * n_hot*row_bytes must fit into the buffer; row_bytes a multiple of 16, table and src_stride 16-byte aligned.
 * The first call allocates a node -> rank array of num_nodes*4 bytes. fg_cache_clear drops the feature side.
 */
fg_status_t fg_cache_fill_features(fg_cache_t* cache, const int32_t* hot_ids_dev, int64_t n_hot, const void* table,
                                   int64_t table_rows, int64_t src_stride, int64_t row_bytes, void* stream);
/*
 * For k < *count_dev (NULL = max_count): rank_out_dev[k] = rank of node ids_dev[k]'s row on the feature side if it
 * was placed and is still intact, else -1 (also for an id outside [0, num_nodes)). *n_found_dev (int64 device, may
 * be NULL) = how many are >= 0. rank_out_dev may be NULL. For tests and monitoring; the loaders below look up inline.
 */
fg_status_t fg_feature_lookup(const fg_cache_t* cache, const int32_t* ids_dev, const int64_t* count_dev, int64_t max_count,
                              int32_t* rank_out_dev, int64_t* n_found_dev, void* stream);
/* The shared buffer (device pointer; *buffer_bytes_out = its size, may be NULL), rows placed on the feature side,
 * and the byte offset of a layer's ring in the buffer (-1 on error). For tests and monitoring. */
const void* fg_cache_buffer(const fg_cache_t* cache, int64_t* buffer_bytes_out);
int64_t fg_cache_feature_rows(const fg_cache_t* cache);
int64_t fg_cache_ring_offset(const fg_cache_t* cache, int32_t layer);

/* Frees everything the cache owns. Synchronises the device first. NULL is accepted. */
fg_status_t fg_cache_destroy(fg_cache_t* cache);
/* Empties all layers (as after create) and drops the feature side, queued on `stream`. */
fg_status_t fg_cache_clear(fg_cache_t* cache, void* stream);
/* Device pointer to the slot table of `layer` ([capacity x dim], row stride dim*sizeof(dtype)); NULL on error. */
const void* fg_cache_table(const fg_cache_t* cache, int32_t layer);
/* Changes the staleness bound for subsequent lookups. */
fg_status_t fg_cache_set_t_stale(fg_cache_t* cache, int32_t t_stale);

/*
 * Stabilization period (Section 4.1.4): lookups of iterations < n_iterations find nothing and updates of those
 * iterations admit nothing (regular mini-batch training); from iteration n_iterations on the cache is active. 0 = none.
 */
fg_status_t fg_cache_set_stabilization(fg_cache_t* cache, int64_t n_iterations);

/*
 * Snapshot for tests and monitoring: every entry a lookup at iteration `iter` would hit, in slot
 * order: nodes_dev[k], slots_dev[k], stamps_dev[k] (each int32[capacity] device, may be NULL),
 * *count_dev (int64 device) = number of entries, *head_dev (int64 device, may be NULL) = ring header.
 * ws_dev: device workspace of at least fg_workspace_bytes(FG_WS_EXPORT, capacity, 0) bytes.
 */
fg_status_t fg_cache_export(const fg_cache_t* cache, int32_t layer, int64_t iter, int32_t* nodes_dev,
                            int32_t* slots_dev, int32_t* stamps_dev, int64_t* count_dev, int64_t* head_dev,
                            void* ws_dev, size_t ws_bytes, void* stream);

/*
 * Launch-shape overrides for measurements (defaults are tuned for MI355X and need no call). Keys:
 * "gather_wg_per_cu", "gather_host_wg_per_cu", "gather_unroll" (1, 2, 4, 8), "gather_nontemporal" (0/1),
 * "aggregate_wg_per_cu", "top_down_walk" (fg_top_down: 1 = its first launch walks the first two blocks down from the seeds, 0 = one layer per launch), "linear_tile" (fp32 GEMM variant: 0 = default, 8 = one task per workgroup with K split over its wavefronts, 32 = panel kernel, 64 / 128 = LDS-tiled kernel with that many rows; bf16 weights: 1064 / 1128 = the 64 x 64 or the 128 x 128 tile). Process-wide, not thread-safe against concurrent launches. Results never depend on them.
 */
fg_status_t fg_set_tuning(const char* key, int64_t value);

typedef enum { FG_WS_LOOKUP_PRUNE = 0, FG_WS_CACHE_UPDATE = 1, FG_WS_EXPORT = 2 } fg_ws_kind_t;
/* Bytes of device workspace the named call needs for a layer of n nodes (0 on a bad argument). */
size_t fg_workspace_bytes(fg_ws_kind_t kind, int64_t n, int64_t reserved);

/*
 * One layer of the top-down pass (Algorithm 1: V_cache = V ∩ C, remove_subgraph(root = V_cache),
 * V_normal = V \ V_cache; Section 5, GPU graph pruning).
 *
 *   cache, layer, iter  cache to look layer `layer` up in at iteration `iter`; cache == NULL: no lookup
 *                       (the seed layer L, the input layer 0, or a run with the cache disabled)
 *   ids_dev[n]          node ids of the layer by position
 *   live_dev[n]         uint8, 1 = still needed after pruning the layers above; NULL = all live.
 *                       Only live nodes are looked up or listed.
 *   row_start_dev[n], row_end_dev[n], col_dev[nnz], n_src
 *                       block `layer` (device); all three NULL for the input layer. row_end is
 *                       MODIFIED: every row that is not normal gets row_end = row_start. col is read only.
 *                       nnz = entries of col (a row whose range leaves [0, nnz] is treated as empty);
 *                       n_src = number of positions of layer-1 (n_src >= n).
 *   live_src_dev[n_src] out, uint8: set to 0 by the call, then 1 at position j of every normal row j and at
 *                       every neighbour position of a normal row (what survives below). NULL without a block;
 *                       NULL with a block = prune only, liveness of the layer below not wanted.
 *   hit_dev[n]          out, uint8 per position: 1 = live and found in the cache (may be NULL if cache == NULL)
 *   hit_pos_dev, hit_slot_dev   out, int32[n]: positions of the hits in ascending order and their cache slots
 *                       (may be NULL if cache == NULL)
 *   normal_pos_dev      out, int32[n]: positions of V_normal (live, not hit) in ascending order
 *   normal_ids_dev      out, int32[n] or NULL: ids_dev[normal_pos[k]] (what the loader needs for layer 0)
 *   counts_dev          out, int64[3] device: n_live, n_hit, n_normal
 *   ws_dev, ws_bytes    device workspace, >= fg_workspace_bytes(FG_WS_LOOKUP_PRUNE, n, 0)
 */
fg_status_t fg_lookup_prune(const fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev, int32_t n,
                            const uint8_t* live_dev, const int32_t* row_start_dev, int32_t* row_end_dev,
                            const int32_t* col_dev, int64_t nnz, int32_t n_src, uint8_t* live_src_dev, uint8_t* hit_dev,
                            int32_t* hit_pos_dev, int32_t* hit_slot_dev, int32_t* normal_pos_dev,
                            int32_t* normal_ids_dev, int64_t* counts_dev, void* ws_dev, size_t ws_bytes, void* stream);

/*
 * fg_lookup_prune for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments without ws_dev / ws_bytes, same
 * kernels, same results. The scratch memory (a class and a slot per position, three counts per workgroup of 1024
 * positions: 5 bytes per position) is a device array built into the library, about 10.5 MB, which every GPU the
 * library runs on holds until the process ends. The call allocates and frees nothing; its first call on a device asks
 * the runtime for the address of that device's copy of the array (no allocation; make that first call outside a capture).
 * n > FG_LOOKUP_PRUNE_STATIC_MAX_N is rejected with FG_ERR_SHAPE. All calls on one GPU share that GPU's array: calls
 * that may overlap on one GPU (different streams, different threads) race; calls on one stream do not. Nothing in the
 * array needs clearing between calls: every byte a call reads it has written itself.
 */
#define FG_LOOKUP_PRUNE_STATIC_MAX_N 2097152
fg_status_t fg_lookup_prune_static(const fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev, int32_t n,
                                   const uint8_t* live_dev, const int32_t* row_start_dev, int32_t* row_end_dev,
                                   const int32_t* col_dev, int64_t nnz, int32_t n_src, uint8_t* live_src_dev,
                                   uint8_t* hit_dev, int32_t* hit_pos_dev, int32_t* hit_slot_dev, int32_t* normal_pos_dev,
                                   int32_t* normal_ids_dev, int64_t* counts_dev, void* stream);

/*
 * The whole top-down pass (fg_lookup_prune for every layer from the seeds down) in one call. Layer by layer the
 * pass is a chain of dependent random reads, and every launch boundary adds to it; here the cache lookups of all
 * layers, which do not depend on liveness, are done in the first launch, where one wavefront per seed also walks the
 * first two blocks down (a seed's neighbours, and their neighbours unless they are cached), so that the liveness of
 * the two layers below the seeds is settled at once; the layers so settled are classified by one launch, and every
 * further layer by one launch that also compacts the lists of the layers above it. Three launches for three layers.
 * Same results as calling fg_lookup_prune layer by layer.
 *
 * layers[0] is the seed layer, layers[i+1] the layer below layers[i]; each entry carries the arguments of
 * fg_lookup_prune for its layer (same meaning, same NULL rules). cache_layer = 0: no lookup for this layer;
 * otherwise the layer of `cache` to look up (1..n_layers of the cache). layers[i].live_src_dev, when given,
 * must be layers[i+1].live_dev. At most 8 layers.
 * ws_dev: >= fg_top_down_workspace_bytes(n_layers, layers) bytes, 16-byte aligned. Its second half carries liveness
 * marks between the launches and must be ALL ZERO when a call starts; every call leaves it all zero. So: zero-fill the
 * workspace once after allocating it, pass the same ws_dev and ws_bytes on every call that uses it, use it for
 * nothing else, and do not let two calls that share it overlap. (A workspace sized for the largest mini-batch serves
 * every smaller one.)
 */
typedef struct fg_top_down_layer {
    int32_t cache_layer;
    int32_t n;
    const int32_t* ids_dev;
    const uint8_t* live_dev;
    const int32_t* row_start_dev;
    int32_t* row_end_dev;
    const int32_t* col_dev;
    int64_t nnz;
    int32_t n_src;
    uint8_t* live_src_dev;
    uint8_t* hit_dev;
    int32_t* hit_pos_dev;
    int32_t* hit_slot_dev;
    int32_t* normal_pos_dev;
    int32_t* normal_ids_dev;
    int64_t* counts_dev;
    const int64_t* n_dev; /* NULL, or the layer's size as a count in device memory (a mini-batch sampled on the device, Section 5:
                             sampling runs ahead of training and nothing waits for its sizes): n, nnz and n_src are then
                             host-side bounds, every array holds that many entries, positions at or beyond
                             min(*n_dev, n) are dead, and the flags of the positions up to n are still written */
} fg_top_down_layer_t;
size_t fg_top_down_workspace_bytes(int32_t n_layers, const fg_top_down_layer_t* layers);
fg_status_t fg_top_down(const fg_cache_t* cache, int64_t iter, int32_t n_layers, const fg_top_down_layer_t* layers,
                        void* ws_dev, size_t ws_bytes, void* stream);

/*
 * Row gather, a bit copy: for k < *count_dev: dst[dst_pos[k], :] = table[src_index[k], :].
 * Serves Load_feature(V_normal^(0)) (Algorithm 1; Section 6, one-sided reads by node id: `table` may be
 * pinned host memory mapped into the device address space) and the cache fetch h_v = C^(l)[v].
 *
 *   table, table_rows, src_stride   source table (device or mapped host), rows, bytes between rows
 *   row_bytes                       bytes copied per row (multiple of 2)
 *   src_index_dev[max_count]        int32 row numbers in the table (node ids or cache slots)
 *   dst_pos_dev[max_count]          int32 destination rows, or NULL for k itself
 *   count_dev, max_count            int64 device count (NULL = max_count) and its host-known upper bound
 *   dst, dst_rows, dst_stride       destination (device), rows, bytes between rows
 *   table_kind                      FG_TABLE_* below: where the rows live and whether they are read once (a hint
 *                                   for the load policy and launch shape only; results do not depend on it)
 * Entries with src_index or dst_pos out of range are skipped. Pointers and strides must be aligned to
 * the largest power of two <= 16 that divides row_bytes.
 */
typedef enum {
    FG_TABLE_HBM_STREAMED = 0, /* big table in HBM, each row read once per call (raw features) */
    FG_TABLE_HOST_MAPPED = 1,  /* table in pinned host memory mapped into the device address space */
    FG_TABLE_HBM_REUSED = 2    /* rows recently written or read again soon (cached embeddings, layer outputs) */
} fg_table_kind_t;

fg_status_t fg_gather(const void* table, int64_t table_rows, int64_t src_stride, int64_t row_bytes,
                      const int32_t* src_index_dev, const int32_t* dst_pos_dev, const int64_t* count_dev,
                      int64_t max_count, void* dst, int64_t dst_rows, int64_t dst_stride, int32_t table_kind,
                      void* stream);

/*
 * fg_gather_aggregate for a block whose columns are given as node ids: col_ids_dev[e] is the table row of the e-th sampled
 * neighbour itself (what src_ids_dev[col_dev[e]] is in fg_gather_aggregate), so the loader does not look positions up.
 * row_ids_dev[n_block_rows] = node id of every row of the block (for the copy of the rows' own features). A sampler that
 * feeds only this loader need not number the input layer at all. Same results as fg_gather_aggregate.
 * cache, n_fetch_layers, fetch_layers: optional (NULL, 0, NULL): the fetch of cached embeddings fg_cache_fetch_all would do
 * for these layers rides along in the same launch (the two jobs are independent; fp32 -> fp32 and fp16 -> bf16 loaders;
 * other type pairs run it as a launch of its own first). fg_fetch_layer_t is declared with fg_cache_fetch_all below.
 */
struct fg_fetch_layer;
fg_status_t fg_gather_aggregate_ids(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_ids_dev,
                                    int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                    int64_t max_rows, const int32_t* row_ids_dev, const void* table, int64_t table_rows,
                                    int64_t src_stride, int32_t dim, fg_dtype_t in_dtype, void* agg, int64_t agg_stride,
                                    fg_dtype_t out_dtype, void* h_self_out, int64_t h_self_stride, int32_t n_self_rows,
                                    const fg_cache_t* cache, int32_t n_fetch_layers, const struct fg_fetch_layer* fetch_layers,
                                    void* stream);

/*
 * Load_feature through the feature side of the bidirectional cache (Section 4.2): fg_gather with node ids as
 * src_index, where the row of a node that fg_feature_lookup would find is read from the shared buffer in HBM
 * instead of from `table`. The result is the same bit copy as fg_gather's; only where the bytes come from differs.
 * table_rows <= the cache's num_nodes; row_bytes must equal the placed rows' size; everything 16-byte aligned.
 * Without a populated feature side this is fg_gather.
 */
fg_status_t fg_gather_features(const fg_cache_t* cache, const void* table, int64_t table_rows, int64_t src_stride,
                               int64_t row_bytes, const int32_t* ids_dev, const int32_t* dst_pos_dev, const int64_t* count_dev,
                               int64_t max_count, void* dst, int64_t dst_rows, int64_t dst_stride, int32_t table_kind,
                               void* stream);

/*
 * Mean aggregation over sampled neighbours (AGG of Eq. 1 with the mean aggregator), for the rows listed:
 *   agg[k, :] = (1/deg) * sum_{e in [row_start[r], row_end[r])} h_src[col[e], :],  r = rows[k], k < *n_rows_dev;
 *   a row without neighbours gives zeros.
 * Sums are carried in fp64 and rounded once to out_dtype.
 *   row_start_dev, row_end_dev [n_block_rows], col_dev[nnz]   the (pruned) block
 *   rows_dev[max_rows]       int32 positions (V_normal, ascending); NULL = 0..count-1
 *   h_src, n_src, src_stride previous-layer embeddings by position (device), rows, byte stride; in_dtype
 *   agg, agg_stride          output [max_rows x dim] compact (row k for rows[k]), any out_dtype; 16-byte aligned
 *   dim * sizeof(in_dtype) must be a multiple of 16.
 */
fg_status_t fg_aggregate(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                         int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                         const void* h_src, int32_t n_src, int64_t src_stride, int32_t dim, fg_dtype_t in_dtype,
                         void* agg, int64_t agg_stride, fg_dtype_t out_dtype, void* stream);

/*
 * Loader fused with the first layer's aggregation: the same mean, taken straight from the feature table without
 * materialising the neighbours' rows (Load_feature and the AGG of Eq. 1 in one pass; every needed table row is
 * still read exactly once per referencing edge, nothing is written but the means):
 *   agg[k, :] = (1/deg) * sum_{e in [row_start[r], row_end[r])} table[src_ids[col[e]], :],  r = rows[k]
 * Arguments as for fg_aggregate, with h_src replaced by
 *   src_ids_dev[n_src]              node id of every position of the input layer
 *   table, table_rows, src_stride   the feature table (device, or host memory mapped into the device address space)
 *   h_self_out, h_self_stride, n_self_rows   optional (NULL to skip): the listed rows' own features, which fg_linear
 *                                   needs, are copied as well: h_self_out[r, :] = table[src_ids[r], :] for r = rows[k]
 *                                   (position r of the input layer is the same node as position r of layer 1)
 * Equal, up to fp64 rounding of the sums, to fg_gather of the input rows followed by fg_aggregate. The top-down
 * call for layer 0 is not needed with it.
 */
fg_status_t fg_gather_aggregate(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                                int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                int64_t max_rows, const int32_t* src_ids_dev, int32_t n_src, const void* table,
                                int64_t table_rows, int64_t src_stride, int32_t dim, fg_dtype_t in_dtype, void* agg,
                                int64_t agg_stride, fg_dtype_t out_dtype, void* h_self_out, int64_t h_self_stride,
                                int32_t n_self_rows, void* stream);

/* fg_gather_aggregate reading through the feature side like fg_gather_features (same arguments and result). */
fg_status_t fg_gather_aggregate_features(const fg_cache_t* cache, const int32_t* row_start_dev, const int32_t* row_end_dev,
                                         const int32_t* col_dev, int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev,
                                         const int64_t* n_rows_dev, int64_t max_rows, const int32_t* src_ids_dev, int32_t n_src,
                                         const void* table, int64_t table_rows, int64_t src_stride, int32_t dim,
                                         fg_dtype_t in_dtype, void* agg, int64_t agg_stride, fg_dtype_t out_dtype,
                                         void* h_self_out, int64_t h_self_stride, int32_t n_self_rows, void* stream);

/*
 * Propagation of a GCN layer in row-normalised form (the paper lists GCN among its models without writing the layer
 * down; on a sampled block only the row's own sampled degree is known, so the graph convolution's self loop and degree
 * normalisation become the mean over the node itself and its sampled neighbours), fp32, for the rows listed:
 *   m[k, :] = (h_src[r, :] + sum_{e in [row_start[r], row_end[r])} h_src[col[e], :]) / (deg + 1),  r = rows[k]
 * The dense part of the layer, act(m . W + b) with W [dim x d_out], is fg_linear with d_in = dim/2, and the mean is
 * written in the form that call reads:
 *   mean_pos_dev[r, 0:dim/2] = m[k, 0:dim/2]     (by position, n_block_rows rows)  -> fg_linear's h_src
 *   mean_cmp_dev[k, 0:dim/2] = m[k, dim/2:dim]   (list order, max_rows rows)       -> fg_linear's agg
 * dim a multiple of 8; other arguments as for fg_aggregate / fg_gather_aggregate.
 */
fg_status_t fg_aggregate_gcn(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz,
                             int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                             const float* h_src, int32_t n_src, int64_t src_stride, int32_t dim, float* mean_pos_dev,
                             float* mean_cmp_dev, void* stream);
fg_status_t fg_gather_aggregate_gcn(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                                    int64_t nnz, int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                    int64_t max_rows, const int32_t* src_ids_dev, int32_t n_src, const float* table,
                                    int64_t table_rows, int64_t src_stride, int32_t dim, float* mean_pos_dev,
                                    float* mean_cmp_dev, void* stream);

/*
 * Dense update of a GraphSAGE-mean layer (phi of Eq. 1; the f_W line of Algorithm 1), for the rows listed:
 *   h_out[r, :] = act( h_src[r, :] . W[0:d_in, :] + agg[k, :] . W[d_in:2*d_in, :] + bias ),  r = rows[k]
 *   act = ReLU if relu != 0, identity otherwise.
 *   h_src (in_dtype; F16 rows are converted to BF16 when w_dtype is BF16), agg (F32 when w_dtype is F32, BF16 when BF16)
 *   W [2*d_in x d_out] row-major, w_dtype F32 or BF16 (bf16 MFMA, fp32 accumulate).
 *   F32: every product of two fp32 values is formed exactly enough for the 1e-5 bar of the path: either by the fp32
 *   matrix instructions, or (the default where the shape allows) from an exact three-way bf16 split of both factors,
 *   six partial products on the bf16 matrix instructions (the dropped ones are below 2^-26 of the product). The
 *   leading partial product has an fp32 running sum of its own, the five small ones share a second one (the roundings
 *   of a running sum are what limits it, and the small products' are 2^-8 of the leading one's); the two are added in
 *   fp64 with the bias and rounded once. Input domain of that kernel: finite values below 2^127 in magnitude (the
 *   split of a larger value overflows to infinity); a nonzero value below 2^-100 may lose its third bf16 term to
 *   underflow, i.e. keeps 16 instead of 24 significant bits (harmless next to larger values of the same row).
 *   bias float[d_out] (device); h_out rows of out_dtype (F32 or BF16) written at position rows[k]
 *   d_in must be a multiple of 4 (8 for 16-bit inputs), d_out a multiple of 4.
 */
fg_status_t fg_linear(const void* h_src, int32_t n_src, int64_t src_stride, fg_dtype_t in_dtype, const void* agg,
                      int64_t agg_stride, const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                      int32_t d_in, int32_t d_out, const void* W, fg_dtype_t w_dtype, const float* bias, int32_t relu,
                      void* h_out, int32_t n_out, int64_t out_stride, fg_dtype_t out_dtype, void* stream);

/*
 * fg_linear with the weights given transposed: Wt is [d_out x 2*d_in] row-major (the weights of one output column are
 * contiguous), bf16 only (FG_ERR_DTYPE otherwise). Same result as fg_linear on the untransposed matrix. This is the layout
 * the bf16 matrix-core kernel reads 16 bytes at a time with nothing to reshuffle on the way into LDS; a caller that keeps
 * its weights across many mini-batches transposes them once (and the backward product dz . W^T takes W itself this way).
 */
fg_status_t fg_linear_wt(const void* h_src, int32_t n_src, int64_t src_stride, fg_dtype_t in_dtype, const void* agg,
                         int64_t agg_stride, const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in,
                         int32_t d_out, const void* Wt, fg_dtype_t w_dtype, const float* bias, int32_t relu, void* h_out,
                         int32_t n_out, int64_t out_stride, fg_dtype_t out_dtype, void* stream);

/*
 * fg_linear for the input layer with Load_feature (Algorithm 1) of the rows' own features folded into the operand load:
 * the own features of output position r are row src_ids_dev[r] of `table` (node ids into the raw feature table, as
 * fg_gather reads them), so that a loader which forms the neighbour means (fg_gather_aggregate* with h_self_out = NULL)
 * need not copy those rows out and this call need not read the copy back:
 *   h_out[r, :] = act( table[src_ids[r], :] . W[0:d_in, :] + agg[k, :] . W[d_in:2*d_in, :] + bias ),  r = rows[k]
 *   table, table_rows, src_stride   device memory (every own row is read once per 32 or 64 output columns: a table
 *                                   in mapped host memory works but is not what this call is for)
 *   src_ids_dev[n_out]              int32, device; entries whose id is outside [0, table_rows) are skipped like
 *                                   positions outside [0, n_out)
 * Everything else, and the result, as for fg_linear on the gathered rows (same kernels, same arithmetic).
 */
fg_status_t fg_linear_ids(const void* table, int32_t table_rows, int64_t src_stride, fg_dtype_t in_dtype,
                          const int32_t* src_ids_dev, const void* agg, int64_t agg_stride, const int32_t* rows_dev,
                          const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in, int32_t d_out, const void* W,
                          fg_dtype_t w_dtype, const float* bias, int32_t relu, void* h_out, int32_t n_out, int64_t out_stride,
                          fg_dtype_t out_dtype, void* stream);


/*
 * fg_aggregate followed by fg_linear for one fp32 GraphSAGE-mean layer (Eq. 1 in one call; same results as the two
 * calls). A layer with few rows, ceil(max_rows/32) * ceil(d_out/32) <= 768 with d_in a multiple of 32 and at most 256
 * (in practice the seed layer), runs as ONE launch that forms the neighbour means while it loads its operands and never
 * writes them; any other shape runs the two calls with the means in agg_ws_dev ([max_rows x d_in] floats, agg_stride
 * bytes between rows, 16-byte aligned; may be NULL when the one-launch form applies).
 * Arguments as for fg_aggregate (block, rows, h_src = H(l-1) by position) and fg_linear (W, bias, relu, h_out).
 */
fg_status_t fg_aggregate_linear(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz,
                                int32_t n_block_rows, const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows,
                                const float* h_src, int32_t n_src, int64_t src_stride, int32_t d_in, int32_t d_out,
                                const float* W, const float* bias, int32_t relu, float* agg_ws_dev, int64_t agg_stride,
                                float* h_out, int32_t n_out, int64_t out_stride, void* stream);

/*
 * Update(C^(l), V_normal^(l), V^(l), h^(l), i, t_stale, p_grad) of Algorithm 1 (Sections 4.1.1, 4.1.2, 4.2).
 * Over the live nodes of the layer (m of them): k = floor(p_grad * m), tau = the gradient norm of rank k
 * (ascending, 0-based; every norm is below tau if k >= m, none if k == 0). Live hits whose norm is not below
 * tau are checked out (mapping entry invalidated); normal nodes (live, not hit) whose norm is below tau are
 * admitted in ascending position order into ring slots head, head+1, ... (mod capacity): their row of h is
 * copied into the table and stamped with `iter`; at most `capacity` per call, the rest are counted as dropped.
 *
 *   ids_dev[n], live_dev[n] (NULL = all live), hit_dev[n]   as given to / produced by fg_lookup_prune
 *   gnorm_dev[n]        float, L2 norm of the loss gradient w.r.t. each node's embedding; finite and >= 0
 *   h_dev, h_stride     embeddings of the layer by position (type = the cache's dtype, width = its dim)
 *   stats_dev           out, int64[4] device or NULL: admitted, evicted_by_gradient, overwritten, dropped_overflow
 *   ws_dev, ws_bytes    device workspace, >= fg_workspace_bytes(FG_WS_CACHE_UPDATE, n, 0)
 * `iter` must not decrease between updates of a layer (FG_ERR_STATE).
 */
fg_status_t fg_cache_update(fg_cache_t* cache, int32_t layer, int64_t iter, const int32_t* ids_dev, int32_t n,
                            const uint8_t* live_dev, const uint8_t* hit_dev, const float* gnorm_dev, float p_grad,
                            const void* h_dev, int64_t h_stride, int64_t* stats_dev, void* ws_dev, size_t ws_bytes,
                            void* stream);

/*
 * The whole last loop of Algorithm 1 ("for l: Update(C^(l), ...)") in one call: the same result as
 * fg_cache_update for each listed layer (each layer at most once, at most 8), with the launches shared by the
 * layers. Fields of a layer as in fg_cache_update; p_grad and iter are common.
 *   ws_dev, ws_bytes    device workspace, >= the sum over the listed layers of
 *                       fg_workspace_bytes(FG_WS_CACHE_UPDATE, layers[i].n, 0); 16-byte aligned
 * Nothing is launched if any layer's arguments are rejected.
 * Access-aware admission (the cache policy "for accuracy and performance" of Section 7.4, which prefers embeddings that
 * save more memory access; the text defines neither the estimate nor the rule, so both are this library's reading): a
 * layer admits at most min(max_admit, capacity) rows per update. If more pass the gradient rule, those with the largest
 * saving_dev[position] (values above 2047 count as 2047) get in, among equal ones the lower positions; the admitted rows
 * are still written in position order from the ring header, and stats_dev[3] counts the rows turned away. saving_dev
 * NULL: all equal, i.e. the first max_admit in position order. One more launch when a layer uses it.
 */
typedef struct fg_update_layer {
    int32_t layer;
    int32_t n;
    const int32_t* ids_dev;
    const uint8_t* live_dev;
    const uint8_t* hit_dev;
    const float* gnorm_dev;
    const void* h_dev;
    int64_t h_stride;
    int64_t* stats_dev;
    const int32_t* saving_dev; /* access-aware admission: estimates by position (fg_access_estimate), or NULL */
    int64_t max_admit;         /* rows this update may admit; 0 = the ring's capacity */
    const int64_t* n_dev;      /* NULL, or the layer's size as a count in device memory (a mini-batch sampled on the device):
                                  n is then its host-side bound, the arrays hold n entries and positions at or beyond
                                  min(*n_dev, n) are ignored; the workspace is sized by n */
} fg_update_layer_t;
fg_status_t fg_cache_update_all(fg_cache_t* cache, int64_t iter, float p_grad, int32_t n_layers,
                                const fg_update_layer_t* layers, void* ws_dev, size_t ws_bytes, void* stream);

/*
 * fg_cache_update_all in two parts, for callers whose gradient norms are known before the embeddings are (norms supplied
 * from outside, as in the benchmark workloads): _select does everything but the row copy (threshold, check-outs,
 * admissions, slots, the cache's index and ring header: it reads ids, live, hit, gnorm, saving and never h_dev), so it can
 * run on another stream while the layers are still being computed; _commit copies the admitted rows from h_dev into
 * their slots. Same descriptors, same iteration and the same workspace (untouched in between) for both calls. Between
 * the two the cache must not be updated again (FG_ERR_STATE). Lookups ordered after _select see the new index, so the next
 * mini-batch may be looked up and pruned before _commit; the rows of its hits must be fetched after _commit. Rows cached
 * before may be fetched in between (fg_cache_fetch_all, fg_gather on fg_cache_table), and _commit must be ordered after
 * those fetches, because a recycled slot's old row is overwritten by it. With raw features placed in the
 * cache's buffer (fg_cache_fill_features) _select must also be ordered after the iteration's feature loads: it advances
 * the rings' written extents, which decide whether a placed feature row is still valid.
 */
fg_status_t fg_cache_update_select(fg_cache_t* cache, int64_t iter, float p_grad, int32_t n_layers,
                                   const fg_update_layer_t* layers, void* ws_dev, size_t ws_bytes, void* stream);
fg_status_t fg_cache_update_commit(fg_cache_t* cache, int64_t iter, int32_t n_layers, const fg_update_layer_t* layers,
                                   void* ws_dev, size_t ws_bytes, void* stream);

/*
 * Neighbour sampling of one block on the device (uniform sampling with a fan-out per layer, Section 7.1; the paper samples
 * on CPU threads, Section 5, so the scheme below is this library's): from the nodes of layer `layer` to block `layer`
 * and the node list of the layer below, over an in-neighbour CSR in device-visible memory.
 * For node v with degree d: slots 0..d-1 if d <= fanout; otherwise f = fanout disjoint strata with integer bounds,
 * stratum j = [floor(j d / f), floor((j + 1) d / f)), draw j = 0..f-1 takes the slot at offset floor(u_j * width_j) of
 * stratum j, and all f slots are moved round the row by the common offset floor(u_f * d), modulo d: f distinct slots,
 * every slot of the row with probability f / d. u_j is the top 53 bits of w(w(w(mix(key), layer), v), j) scaled to [0, 1),
 * w(k, c) = mix(k + (c + 1) * 0x9E3779B97F4A7C15) and mix the SplitMix64 output function.
 * The row keeps the neighbours at those slots in the order of j, without v itself and without repeats. The layer below is this
 * layer's nodes followed by the neighbours not among them, each once, in order of first occurrence (rows in order, slots
 * in order). The result is a pure function of the arguments.
 *   indptr_dev [num_nodes + 1] int64, indices_dev [num_edges] int32   in-neighbours of v: indices[indptr[v] .. indptr[v+1])
 *   ids_dev [max_rows], n_dev, max_rows   distinct node ids of the layer; device-side count (NULL = max_rows) and its
 *                                         host-side bound; fanout in 1..32
 *   row_start_dev, row_end_dev [max_rows] out: rows back to back, rows at and beyond the count are empty
 *   col_dev [max_rows * fanout]           out: positions in the layer below
 *   col_ids_dev [max_rows * fanout]       out, optional (NULL): the same columns as node ids
 *   ids_below_dev [max_below]             out: node ids of the layer below; max_below >= max_rows, and at least
 *                                         max_rows * (1 + fanout) to be safe for every input: if counts_dev[0] comes out
 *                                         larger than max_below the list was cut and the block must be discarded
 *   counts_dev [2] int64                  out: nodes of the layer below, edges of the block
 *   ws_dev, ws_bytes                      device workspace, >= fg_sample_block_workspace_bytes(max_rows, fanout) (0 for
 *                                         sizes the call rejects); 16-byte aligned
 * Six launches on `stream`, no host synchronisation. Node ids outside [0, num_nodes) get empty rows.
 */
size_t fg_sample_block_workspace_bytes(int64_t max_rows, int32_t fanout);
fg_status_t fg_sample_block(const int64_t* indptr_dev, const int32_t* indices_dev, int64_t num_nodes, int64_t num_edges,
                            const int32_t* ids_dev, const int64_t* n_dev, int64_t max_rows, int32_t fanout, uint64_t key,
                            int32_t layer, int32_t* row_start_dev, int32_t* row_end_dev, int32_t* col_dev, int32_t* col_ids_dev,
                            int32_t* ids_below_dev, int64_t max_below, int64_t* counts_dev, void* ws_dev, size_t ws_bytes,
                            void* stream);

/*
 * The transpose of a sampled block, which fg_layer_backward walks: for every position j of the layer below, the rows that
 * sampled it, in ascending order, back to back (t_row[t_start[j] .. t_end[j])). Built from the block as given: call it on
 * the sampled block, before the top-down pass prunes rows.
 *   row_start_dev, row_end_dev [max_rows], col_dev [max_nnz]   the block; n_dev: device-side row count (NULL = max_rows)
 *   n_src_dev, max_src                     device-side node count of the layer below (NULL = max_src) and its bound;
 *                                          columns outside [0, count) are ignored
 *   t_start_dev, t_end_dev [max_src], t_row_dev [max_nnz]      out; positions at and beyond the count get empty lists
 *   ws_dev, ws_bytes                       device workspace, >= fg_transpose_block_workspace_bytes(max_src); 16-byte aligned
 * Six launches, no host synchronisation; the result does not depend on the order in which threads run.
 */
size_t fg_transpose_block_workspace_bytes(int64_t max_src);
fg_status_t fg_transpose_block(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev,
                               const int64_t* n_dev, int64_t max_rows, const int64_t* n_src_dev, int64_t max_src, int64_t max_nnz,
                               int32_t* t_start_dev, int32_t* t_end_dev, int32_t* t_row_dev, void* ws_dev, size_t ws_bytes,
                               void* stream);

/*
 * The estimate the access-aware admission ranks by: the rows read to produce each node's embedding in this mini-batch,
 * counted along the pruned block like a tree (no credit for neighbours shared with other rows). out[j] = 1 for a node
 * served from the cache (hit_dev[j] != 0); otherwise below[j] + the sum of below[col[c]] over the neighbours left in row
 * j, with below == NULL meaning the input layer (every row one read). Saturates at 2047. Call it bottom-up, layer 1
 * first, after the top-down pass has pruned the blocks.
 *   row_start_dev, row_end_dev [n], col_dev [nnz]   the layer's block after pruning (columns: positions in the layer below)
 *   hit_dev [n]                                      the layer's hit flags, or NULL (no cache at this layer)
 *   below_dev [n_src]                                estimates of the layer below by position, or NULL; n_src >= n
 *   out_dev [n]                                      int32 estimates by position
 * All pointers device memory; one launch, no host synchronisation.
 */
fg_status_t fg_access_estimate(const int32_t* row_start_dev, const int32_t* row_end_dev, const int32_t* col_dev, int64_t nnz,
                               int32_t n, const uint8_t* hit_dev, const int32_t* below_dev, int32_t n_src, int32_t* out_dev,
                               void* stream);

/*
 * The fetch of cached embeddings (h_v = C^(l)[v], Algorithm 1) for every hit of every listed layer in one launch:
 * the same result as fg_gather(fg_cache_table(cache, layer), capacity, ..., hit_slot, hit_pos, n_hit, ..., h) per
 * layer. At most 8 layers.
 *   hit_slot_dev, hit_pos_dev [max_hits], n_hit_dev   the hit lists and their device-side count (NULL = max_hits)
 *                                                     as produced by fg_lookup_prune / fg_top_down
 *   h_dev, h_rows, h_stride                           embeddings of the layer by position (the cache's dtype and width),
 *                                                     rows, byte stride; 16-byte aligned
 * Entries with a slot or position out of range are skipped.
 */
typedef struct fg_fetch_layer {
    int32_t layer;
    const int32_t* hit_slot_dev;
    const int32_t* hit_pos_dev;
    const int64_t* n_hit_dev;
    int64_t max_hits;
    void* h_dev;
    int64_t h_rows;
    int64_t h_stride;
} fg_fetch_layer_t;
fg_status_t fg_cache_fetch_all(const fg_cache_t* cache, int32_t n_layers, const fg_fetch_layer_t* layers, void* stream);

/*
 * ---- Backward pass as far as the embedding gradients (Algorithm 1: loss, loss.backward(); Section 4.1.1) ----
 * The norms of dL/dh^(l) are the gradient criterion of the cache: fg_row_norms of what fg_layer_backward produces
 * is the gnorm_dev of fg_cache_update. Gradients are fp32 throughout; sums in fp64.
 *
 * fg_softmax_xent_grad: dh[i, c] = (softmax(h[i, :])[c] - [c == labels[i]]) / n, the gradient of the mean softmax
 * cross-entropy over the n seed rows (the paper trains node classifiers and does not fix the loss further).
 * A label outside [0, d) leaves out the subtraction for that row.
 */
fg_status_t fg_softmax_xent_grad(const float* h_dev, int64_t h_stride, const int32_t* labels_dev, int32_t n, int32_t d,
                                 float* dh_dev, int64_t dh_stride, void* stream);
/* norms_dev[i] = sqrt(sum_c x[i, c]^2) for i < n (the magnitude of an embedding's gradient, Section 4.1.1). */
fg_status_t fg_row_norms(const float* x_dev, int64_t x_stride, int32_t n, int32_t d, float* norms_dev, void* stream);
/*
 * Gradient with respect to the inputs of one GraphSAGE-mean layer (the transpose of fg_aggregate + fg_linear):
 *   dz[k, :] = dh[r, :] * (h[r, :] > 0), r = rows[k]   (h = the layer's output; NULL = no activation, the last layer)
 *   [d_self ‖ d_agg][k, :] = dz[k, :] . W^T            (W as given to fg_linear: [2*d_in x d_out])
 *   dh_src[j, :] = [j = rows[k] for some k] d_self[k, :] + sum over the rows r = rows[k] that sampled j of d_agg[k, :] / deg(r)
 * for every position j < n_src of the layer below (zeros where nothing arrives). Rows that were fetched from the
 * cache or pruned are not in `rows` and pass nothing down.
 *   dh_dev, dh_stride, h_dev, h_stride   dL/dH(l) and H(l) by position, n rows of d_out floats
 *   rows_dev, n_rows_dev, max_rows       V_normal of the layer as produced by the top-down pass (max_rows <= n)
 *   live_dev, hit_dev [n]                the layer's flags (NULL = all live / no hits): position j is in `rows` iff live and not hit
 *   row_start_dev, row_end_dev [n]       block l after pruning: deg(r) = row_end[r] - row_start[r]; rows not in `rows` must have deg 0
 *   t_start_dev, t_end_dev [n_src], t_row_dev [nnz]   the transpose of the sampled block: the rows that sampled position j are
 *                                        t_row[t_start[j] .. t_end[j]) (of the block before pruning; pruned rows are skipped by deg 0)
 *   W, d_in, d_out                       the layer's weights; d_in a multiple of 4, d_out of 8
 *   dh_src_dev, dh_src_stride            out: dL/dH(l-1) by position [n_src x d_in], 16-byte aligned
 *   norms_src_dev                        out, float[n_src] or NULL: the L2 norm of every row of dh_src (what fg_row_norms would give)
 *   ws_dev, ws_bytes                     device workspace >= fg_layer_backward_workspace_bytes(n, max_rows, d_in, d_out), 16-byte aligned
 * No atomics: every output row has one writer, so results do not depend on scheduling.
 */
size_t fg_layer_backward_workspace_bytes(int32_t n, int64_t max_rows, int32_t d_in, int32_t d_out);
fg_status_t fg_layer_backward(const float* dh_dev, int64_t dh_stride, const float* h_dev, int64_t h_stride, int32_t n,
                              const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows, const uint8_t* live_dev,
                              const uint8_t* hit_dev, const int32_t* row_start_dev, const int32_t* row_end_dev,
                              const int32_t* t_start_dev, const int32_t* t_end_dev, const int32_t* t_row_dev, int64_t nnz,
                              int32_t n_src, int32_t d_in, int32_t d_out, const float* W, float* dh_src_dev,
                              int64_t dh_src_stride, float* norms_src_dev, void* ws_dev, size_t ws_bytes, void* stream);

/*
 * The same for a GCN layer in the form of fg_aggregate_gcn + fg_linear (Section 7.5: the method carries over to other
 * layer types; m_r = (h_r + sum of the sampled neighbours' rows) / (deg(r) + 1), one weight matrix W [d_in x d_out]):
 *   dz as above,  dm[k, :] = dz[k, :] . W^T,
 *   dh_src[j, :] = [j = rows[k] for some k] dm[k, :] / (deg(j) + 1) + sum over the rows r = rows[k] that sampled j of dm[k, :] / (deg(r) + 1)
 * Arguments as for fg_layer_backward; d_in a multiple of 4, d_out of 8.
 */
size_t fg_layer_backward_gcn_workspace_bytes(int32_t n, int64_t max_rows, int32_t d_in, int32_t d_out);
fg_status_t fg_layer_backward_gcn(const float* dh_dev, int64_t dh_stride, const float* h_dev, int64_t h_stride, int32_t n,
                                  const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows, const uint8_t* live_dev,
                                  const uint8_t* hit_dev, const int32_t* row_start_dev, const int32_t* row_end_dev,
                                  const int32_t* t_start_dev, const int32_t* t_end_dev, const int32_t* t_row_dev, int64_t nnz,
                                  int32_t n_src, int32_t d_in, int32_t d_out, const float* W, float* dh_src_dev,
                                  int64_t dh_src_stride, float* norms_src_dev, void* ws_dev, size_t ws_bytes, void* stream);
/*
 * fg_layer_backward for the mixed-precision setting of Section 7.4's largest runs (embeddings and weights in bf16). The
 * paper does not say where the backward pass rounds; the reading taken mirrors the forward product: both operands of
 * dz . W^T are bf16 (dz rounded to nearest even after the mask, W as stored), products and sums in fp32, and the gradients
 * themselves (dh, dh_src, the norms) stay fp32.
 *   h_dev, h_stride   H(l) by position in bf16 (NULL = no activation);  W  bf16 [2*d_in x d_out], 16-byte aligned
 *   d_in a multiple of 8, d_out of 16; everything else as for fg_layer_backward.
 */
size_t fg_layer_backward_bf16_workspace_bytes(int32_t n, int64_t max_rows, int32_t d_in, int32_t d_out);
fg_status_t fg_layer_backward_bf16(const float* dh_dev, int64_t dh_stride, const void* h_dev, int64_t h_stride, int32_t n,
                                   const int32_t* rows_dev, const int64_t* n_rows_dev, int64_t max_rows, const uint8_t* live_dev,
                                   const uint8_t* hit_dev, const int32_t* row_start_dev, const int32_t* row_end_dev,
                                   const int32_t* t_start_dev, const int32_t* t_end_dev, const int32_t* t_row_dev, int64_t nnz,
                                   int32_t n_src, int32_t d_in, int32_t d_out, const void* W, float* dh_src_dev,
                                   int64_t dh_src_stride, float* norms_src_dev, void* ws_dev, size_t ws_bytes, void* stream);

/*
 * Gradient with respect to the weights of one GraphSAGE-mean layer, over the computed rows (dz as in fg_layer_backward):
 *   dw[a, c] = sum_k x[k, a] * dz[k, c],  x[k, :] = [h_src[rows[k], :] ‖ agg[k, :]]   ([2*d_in x d_out], the layout of W)
 *   db[c]    = sum_k dz[k, c]                                                          (db_dev may be NULL)
 * h_src, agg, rows as given to fg_linear for this layer in the forward pass; dh, h (NULL = no activation) by position,
 * n rows. Every fp32 product is formed exactly, on the bf16 matrix cores from three-way splits of both operands as in
 * fg_linear (or on the fp32 matrix instructions where an operand ends beyond 4 GB); fp32 sums within a slice of the rows,
 * fp64 across slices; the slicing depends only on max_rows and the number of rows, so results do not depend on
 * scheduling. Input domain as for fg_linear.
 *   ws_dev, ws_bytes    device workspace >= fg_layer_backward_weights_workspace_bytes(max_rows, d_in, d_out), 16-byte aligned
 */
size_t fg_layer_backward_weights_workspace_bytes(int64_t max_rows, int32_t d_in, int32_t d_out);
fg_status_t fg_layer_backward_weights(const float* h_src_dev, int32_t n_src, int64_t src_stride, const float* agg_dev,
                                      int64_t agg_stride, const float* dh_dev, int64_t dh_stride, const float* h_dev,
                                      int64_t h_stride, int32_t n, const int32_t* rows_dev, const int64_t* n_rows_dev,
                                      int64_t max_rows, int32_t d_in, int32_t d_out, float* dw_dev, float* db_dev,
                                      void* ws_dev, size_t ws_bytes, void* stream);

/*
 * For a GCN layer the same call serves: its input rows are the propagated rows m_r, which fg_aggregate_gcn leaves as a
 * by-position first half and a list-order second half; give those as h_src and agg with d_in = half the layer's input
 * width and dw comes out as [d_in x d_out], the layout of the layer's W.
 *
 * fg_layer_backward_weights_bf16: the mixed-precision setting. agg and h are bf16, h_src is fp32, fp16 or bf16 (src_dtype;
 * rounded to bf16 as the forward product rounds it); dz is rounded to bf16 before it enters x^T dz, the bias gradient
 * sums the unrounded dz. With both operands bf16 the contraction over the computed rows runs on the bf16 matrix cores:
 * one launch writes x and dz transposed (the contraction index contiguous) into the workspace, the forward matrix-core
 * kernel multiplies them with fp32 sums over all rows (its loop stops at the device-side row count), a last launch adds
 * up the bias gradient's partial sums in fp64. d_in and d_out multiples of 8; pointers and strides 4-byte aligned, dw and
 * db 16-byte. Deterministic.
 *   ws_dev, ws_bytes    device workspace >= fg_layer_backward_weights_bf16_workspace_bytes(max_rows, d_in, d_out), 16-byte aligned
 */
size_t fg_layer_backward_weights_bf16_workspace_bytes(int64_t max_rows, int32_t d_in, int32_t d_out);
fg_status_t fg_layer_backward_weights_bf16(const void* h_src_dev, int32_t n_src, int64_t src_stride, fg_dtype_t src_dtype,
                                           const void* agg_dev, int64_t agg_stride, const float* dh_dev, int64_t dh_stride,
                                           const void* h_dev, int64_t h_stride, int32_t n, const int32_t* rows_dev,
                                           const int64_t* n_rows_dev, int64_t max_rows, int32_t d_in, int32_t d_out,
                                           float* dw_dev, float* db_dev, void* ws_dev, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FRESHGNN_H */
