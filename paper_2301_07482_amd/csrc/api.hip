// Error reporting, version and workspace sizing of the C ABI.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "common.h"

static thread_local char g_err[512] = "";

void fg_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

void fg_clear_error() { g_err[0] = 0; }

size_t fg_ws_lookup_prune_bytes(int64_t n);
size_t fg_ws_cache_update_bytes(int64_t n);
size_t fg_ws_export_bytes(int64_t capacity);

static int64_t g_tune[FG_TUNE_COUNT] = {16, 4, 1, 1, 32, 0, 1};
static const char* const g_tune_names[FG_TUNE_COUNT] = {"gather_wg_per_cu", "gather_host_wg_per_cu", "gather_unroll",
                                                        "gather_nontemporal", "aggregate_wg_per_cu", "linear_tile",
                                                        "top_down_walk"};

int64_t fg_tuning(fg_tune_id id) { return g_tune[id]; }

extern "C" fg_status_t fg_set_tuning(const char* key, int64_t value) {
    if (!key) FG_FAIL(FG_ERR_INVALID_ARG, "fg_set_tuning: key is NULL");
    if (value < 0 || value > 4096) FG_FAIL(FG_ERR_INVALID_ARG, "fg_set_tuning: value %lld out of range", (long long)value);
    for (int i = 0; i < FG_TUNE_COUNT; ++i) {
        if (strcmp(key, g_tune_names[i]) == 0) {
            if (value == 0 && i != FG_TUNE_GATHER_NONTEMPORAL && i != FG_TUNE_LINEAR_TILE && i != FG_TUNE_TOP_DOWN_WALK) FG_FAIL(FG_ERR_INVALID_ARG, "fg_set_tuning: %s must be positive", key);
            g_tune[i] = value;
            return FG_OK;
        }
    }
    FG_FAIL(FG_ERR_INVALID_ARG, "fg_set_tuning: unknown key '%s'", key);
}

extern "C" const char* fg_last_error(void) { return g_err; }

extern "C" int32_t fg_version(void) { return 301; }  // 0.3.1: fg_linear_ids; 0.3.0: device-side layer sizes (two structs grew a field), backward for GCN and mixed precision, fg_linear_wt, fg_lookup_prune_static

extern "C" size_t fg_workspace_bytes(fg_ws_kind_t kind, int64_t n, int64_t reserved) {
    (void)reserved;
    if (n < 0) return 0;
    switch (kind) {
        case FG_WS_LOOKUP_PRUNE: return fg_ws_lookup_prune_bytes(n);
        case FG_WS_CACHE_UPDATE: return fg_ws_cache_update_bytes(n);
        case FG_WS_EXPORT: return fg_ws_export_bytes(n);
        default: return 0;
    }
}
