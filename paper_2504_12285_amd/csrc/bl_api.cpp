/* Host-only entry points of the BitLinear library: sizes, names, version. */
#include "bl_host.h"

#include <atomic>

extern "C" int bl_version(void) { return 100; }

extern "C" const char* bl_status_str(int status) {
    switch (status) {
        case BL_OK: return "BL_OK";
        case BL_ERR_NULL: return "BL_ERR_NULL: a required pointer is NULL";
        case BL_ERR_SHAPE: return "BL_ERR_SHAPE: M/N/K out of range or not a permitted multiple";
        case BL_ERR_LAYOUT: return "BL_ERR_LAYOUT: unknown packed layout";
        case BL_ERR_ALIGN: return "BL_ERR_ALIGN: pointer not aligned as required";
        case BL_ERR_VALUE: return "BL_ERR_VALUE: unknown in_kind or op id";
        case BL_ERR_HIP: return "BL_ERR_HIP: a HIP call or kernel launch failed";
        case BL_ERR_WORKSPACE: return "BL_ERR_WORKSPACE: workspace required but NULL";
        default: return "unknown bl_status";
    }
}

extern "C" size_t bl_packed_bytes(int64_t N, int64_t K, int layout) {
    if (!bl_shape_ok(N, K)) return 0;
    if (layout == BL_LAYOUT_TRIT5) return (size_t)(bl_npad(N) * bl_kpad5(K) / 5);
    if (layout == BL_LAYOUT_KMAJOR) return (size_t)(K * ((N + 63) / 64 * 16));
    if (layout != BL_LAYOUT_ROWMAJOR && layout != BL_LAYOUT_K16) return 0;
    return (size_t)(bl_npad(N) * bl_kpad(K) / 4);
}

extern "C" int64_t bl_padded_k(int64_t K) { return K >= 1 && K <= BL_MAX_DIM ? bl_kpad(K) : 0; }

extern "C" size_t bl_workspace_bytes(int op, int64_t M, int64_t N, int64_t K) {
    (void)N;
    (void)K;
    switch (op) {
        case BL_OP_PACK: return BL_PACK_PARTIALS * sizeof(double);
        case BL_OP_GEMV:
        case BL_OP_GEMM: return M > 0 ? (size_t)((M * 4 + 255) / 256 * 256) : 0;
        default: return 0;
    }
}

static std::atomic<int> g_forced_decode_path{0};
int bl_forced_decode_path(void) { return g_forced_decode_path.load(std::memory_order_relaxed); }
extern "C" bl_status bl_debug_force_path(int path) {
    if (path < 0 || path > 3) return BL_ERR_VALUE;
    g_forced_decode_path.store(path, std::memory_order_relaxed);
    return BL_OK;
}

/* Measurement hook: where the prefill tile kernel leaves the clock counts of its workgroup 0. */
static std::atomic<int64_t*> g_clock_stamps{nullptr};
int64_t* bl_clock_stamps(void) { return g_clock_stamps.load(std::memory_order_relaxed); }
extern "C" bl_status bl_debug_clock_stamps(int64_t* stamps) {
    if (!bl_aligned(stamps, 8)) return BL_ERR_ALIGN;
    g_clock_stamps.store(stamps, std::memory_order_relaxed);
    return BL_OK;
}
