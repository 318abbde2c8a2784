/* Internal host-side helpers: argument checks shared by the entry points. */
#pragma once
#include <stdint.h>

#include "bitlinear.h"

#define BL_PACK_PARTIALS 1024          /* fp64 partial sums used by bl_pack_ternary */
#define BL_NOALLOC_MAX_M 16384          /* rows bl_gemm_w158a8_noalloc accepts        */
#define BL_MAX_DIM ((int64_t)1 << 24)  /* upper bound on M, N and K                 */

static inline bool bl_shape_ok(int64_t N, int64_t K) {
    return N >= 1 && K >= 1 && N <= BL_MAX_DIM && K <= BL_MAX_DIM;
}
/* Padded sizes of the packed matrix and of the quantised activations (bitlinear.h, PACKED LAYOUTS). */
static inline int64_t bl_kpad(int64_t K) { return (K + 63) / 64 * 64; }
static inline int64_t bl_npad(int64_t N) { return (N + 3) / 4 * 4; }
/* Five-per-byte form: rows of ceil(K/80)*80 weights = a whole number of 16-byte loads. */
static inline int64_t bl_kpad5(int64_t K) { return (K + 79) / 80 * 80; }
static inline bool bl_shape_unpadded(int64_t N, int64_t K) { return N % 4 == 0 && K % 64 == 0; }
static inline bool bl_aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

/* Test hook (bl_debug_force_path): which decode kernel bl_gemv_launch_group takes.
 * 0 = the measured default, 1 = dot4 kernel where it applies, 2 = row-resident matrix-core
 * kernel, 3 = streaming panel kernel where it applies.  Process-wide, atomic. */
int bl_forced_decode_path(void);
/* Measurement hook (bl_debug_clock_stamps): device buffer for the clock counts of the prefill
 * tile kernel, or NULL (the default).  Process-wide, atomic. */
int64_t* bl_clock_stamps(void);

/* One product of a table walked by the TABLE form of bl_gemm_tile256 (device memory). */
struct bl_tile_item {
    const uint8_t* packed;
    const int8_t* q;
    const int32_t* rowsum;
    const float* beta;
    const float* scale;       /* NULL: y is not wanted */
    const float* residual;
    int32_t* acc;
    float* y;
    int N, K;                 /* K: the padded row length, a multiple of 128 */
};

/* Launch of that table walk (bl_gemm.hip) for the batched streamed decode (bl_stream.hip). */
int bl_gemm_table_blocks(void);
bl_status bl_gemm_table_launch(const bl_tile_item* items, const int* tile0, int nitems, int total_tiles, int M,
                               int blocks, const int* wg_start, const int* tile_list, bl_stream s);
