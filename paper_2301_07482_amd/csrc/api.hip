// Error reporting, version and workspace sizing of the C ABI.
#include <stdarg.h>
#include <stdio.h>

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

extern "C" const char* fg_last_error(void) { return g_err; }

extern "C" int32_t fg_version(void) { return 100; }

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
