/* Decode-side W1.58A8 product (Section 5.1 of the BitNet b1.58 2B4T report):
 * acc[m][n] = sum_k q[m][k] * Wt[n][k] for small token counts, streaming the
 * 2-bit packed weights from HBM exactly once with 128-bit loads.
 *
 * Arithmetic identity used on chip (exact in int32): with codes c = Wt + 1,
 *   sum_k Wt*q = sum_k c*q - sum_k q .
 * A packed word is never shifted into place: the four bit-pair levels of a
 * word are isolated by masks only (the top level by one shift), multiplied by
 * the matching activation bytes with v_dot4_i32_i8 into four accumulators that
 * carry the factors 1, 4, 16, 16, and recombined once per row with exact
 * shifts.  Partial sums are reduced across lanes with DPP row operations and
 * across the waves of a workgroup through LDS.
 */
#include <stdlib.h>

#include "bl_device.h"
#include "bl_host.h"

/* Activation staging shared by the decode kernels.  LDS holds, for token m and
 * 64-wide k chunk c, sixteen dwords indexed [s][d]: the activation bytes that
 * pair with bit-pair level s of packed word d of the chunk.
 *   layout 1: level s of word d holds k = 16d+4s+{0..3} -> natural dword 4d+s.
 *   layout 0: level s of word d holds k = 16d+{s,4+s,8+s,12+s} -> byte transpose.
 * Also accumulates rowsum[m] = sum_k q[m][k] into LDS (sq). */
template <int LAYOUT>
__device__ __forceinline__ void bl_stage_q(const int8_t* __restrict__ q, int M, int K, int* __restrict__ Q,
                                           int* __restrict__ sq, int tid, int nthreads) {
    const int groups = K / 16;  /* 16-byte groups per token */
    const int nchunks = K / 64;
    for (int u = tid; u < M * groups; u += nthreads) {
        const int m = u / groups, c16 = u - m * groups;
        const uint4 v = *(const uint4*)(q + (int64_t)m * K + (int64_t)c16 * 16);
        uint32_t a0 = v.x, a1 = v.y, a2 = v.z, a3 = v.w;
        int part = __builtin_amdgcn_sdot4((int)a0, 0x01010101, 0, false);
        part = __builtin_amdgcn_sdot4((int)a1, 0x01010101, part, false);
        part = __builtin_amdgcn_sdot4((int)a2, 0x01010101, part, false);
        part = __builtin_amdgcn_sdot4((int)a3, 0x01010101, part, false);
        if (LAYOUT == 0) bl_transpose4x4(a0, a1, a2, a3);
        const int chunk = c16 >> 2, d = c16 & 3;
        int* dst = Q + ((m * nchunks + chunk) * 16 + d);
        dst[0] = (int)a0;
        dst[4] = (int)a1;
        dst[8] = (int)a2;
        dst[12] = (int)a3;
        atomicAdd(&sq[m], part);
    }
}

/* VALU path, M <= 4 tokens.  G lanes share one weight row; a wave covers
 * R = 64/G rows x (G*64) k per step; the waves of a block split the k steps. */
template <int M, int G, int LAYOUT>
__global__ __launch_bounds__(512) void bl_gemv_dot4(const bl_v4i* __restrict__ packed, const int8_t* __restrict__ q,
                                                    const float* __restrict__ beta, const float* __restrict__ scale,
                                                    int N, int K, int32_t* __restrict__ acc, float* __restrict__ y) {
    extern __shared__ int lds[];
    constexpr int R = 64 / G;
    const int nchunks = K / 64;
    int* Q = lds;                      /* M*K/4 dwords */
    int* sq = Q + M * (K / 4);         /* M           */
    int* red = sq + M;                 /* nw*R*M      */
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, nw = blockDim.x >> 6;
    const int r = lane / G, g = lane % G;
    const int n = blockIdx.x * R + r;
    const bool row_ok = n < N;
    const bl_v4i* wrow = packed + (int64_t)(row_ok ? n : 0) * nchunks;

    if (tid < M) sq[tid] = 0;
    __syncthreads();
    bl_stage_q<LAYOUT>(q, M, K, Q, sq, tid, blockDim.x);
    __syncthreads();

    int A[M][4];
#pragma unroll
    for (int m = 0; m < M; ++m) A[m][0] = A[m][1] = A[m][2] = A[m][3] = 0;

    for (int chunk = w * G + g; chunk < nchunks; chunk += nw * G) {
        bl_v4i p = {0, 0, 0, 0};
        if (row_ok) p = __builtin_nontemporal_load(wrow + chunk);
        const uint32_t pw[4] = {(uint32_t)p[0], (uint32_t)p[1], (uint32_t)p[2], (uint32_t)p[3]};
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const bl_v4i* Qc = (const bl_v4i*)(Q + (m * nchunks + chunk) * 16);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bl_v4i qs = Qc[s];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t lv = s == 0 ? (pw[d] & 0x03030303u)
                                      : s == 1 ? (pw[d] & 0x0C0C0C0Cu)
                                      : s == 2 ? (pw[d] & 0x30303030u)
                                               : ((pw[d] >> 2) & 0x30303030u);
                    A[m][s] = __builtin_amdgcn_sdot4((int)lv, qs[d], A[m][s], false);
                }
            }
        }
    }

#pragma unroll
    for (int m = 0; m < M; ++m) {
        int v = A[m][0] + (A[m][1] >> 2) + ((A[m][2] + A[m][3]) >> 4);
        v = bl_group_sum<G>(v);
        if (g == 0) red[(w * R + r) * M + m] = v;
    }
    __syncthreads();
    if (tid < R * M) {
        const int m = tid / R, rr = tid % R;
        const int nn = blockIdx.x * R + rr;
        if (nn < N) {
            int v = -sq[m];
            for (int i = 0; i < nw; ++i) v += red[(i * R + rr) * M + m];
            if (acc) acc[(int64_t)m * N + nn] = v;
            if (y) y[(int64_t)m * N + nn] = (float)v * (*beta * scale[m]);
        }
    }
}

static int bl_env_int(const char* name, int dflt) {
    const char* e = getenv(name);
    return e && *e ? atoi(e) : dflt;
}

template <int M, int G>
static bl_status launch_dot4(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                             const float* scale, int N, int K, int32_t* acc, float* y, int nw, hipStream_t st) {
    constexpr int R = 64 / G;
    const unsigned grid = (unsigned)((N + R - 1) / R);
    const size_t lds = (size_t)(M * (K / 4) + M + nw * R * M) * sizeof(int);
    if (lds > 64 * 1024) return BL_ERR_SHAPE;
    if (layout == 0)
        bl_gemv_dot4<M, G, 0><<<grid, nw * 64, lds, st>>>((const bl_v4i*)packed, q, beta, scale, N, K, acc, y);
    else
        bl_gemv_dot4<M, G, 1><<<grid, nw * 64, lds, st>>>((const bl_v4i*)packed, q, beta, scale, N, K, acc, y);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

template <int M>
static bl_status launch_dot4_g(int G, const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                               const float* scale, int N, int K, int32_t* acc, float* y, int nw, hipStream_t st) {
    switch (G) {
        case 4: return launch_dot4<M, 4>(packed, beta, layout, q, scale, N, K, acc, y, nw, st);
        case 8: return launch_dot4<M, 8>(packed, beta, layout, q, scale, N, K, acc, y, nw, st);
        default: return launch_dot4<M, 16>(packed, beta, layout, q, scale, N, K, acc, y, nw, st);
    }
}

bl_status bl_gemm_dispatch(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                           const float* scale, const int32_t* rowsum, int64_t M, int64_t N, int64_t K,
                           int32_t* acc, float* y, void* workspace, hipStream_t st);

extern "C" bl_status bl_gemv_w158a8(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                                    const float* scale, const int32_t* rowsum, int64_t M, int64_t N, int64_t K,
                                    int32_t* acc, float* y, void* workspace, bl_stream s) {
    if (!packed || !beta || !q) return BL_ERR_NULL;
    if (!acc && !y) return BL_ERR_NULL;
    if (y && !scale) return BL_ERR_NULL;
    if (M < 1 || M > 64 || !bl_shape_ok(N, K)) return BL_ERR_SHAPE;
    if (layout != BL_LAYOUT_ROWMAJOR && layout != BL_LAYOUT_K16) return BL_ERR_LAYOUT;
    if (!bl_aligned(packed, 16) || !bl_aligned(q, 16) || !bl_aligned(acc, 4) || !bl_aligned(y, 4) ||
        !bl_aligned(scale, 4) || !bl_aligned(beta, 4) || !bl_aligned(rowsum, 4))
        return BL_ERR_ALIGN;
    hipStream_t st = (hipStream_t)s;
    if (M > 4 || K > 8192)
        return bl_gemm_dispatch(packed, beta, layout, q, scale, rowsum, M, N, K, acc, y, workspace, st);

    const int nchunks = (int)(K / 64);
    int G = bl_env_int("BL_GEMV_G", 8);
    if (G != 4 && G != 8 && G != 16) G = 8;
    const int steps = (nchunks + G - 1) / G;
    int nw = bl_env_int("BL_GEMV_NW", 0);
    if (nw <= 0) nw = steps < 8 ? steps : (steps + 1) / 2 <= 8 ? (steps + 1) / 2 : 8;
    if (nw > 8) nw = 8;
    if (nw < 1) nw = 1;
    switch ((int)M) {
        case 1: return launch_dot4_g<1>(G, packed, beta, layout, q, scale, (int)N, (int)K, acc, y, nw, st);
        case 2: return launch_dot4_g<2>(G, packed, beta, layout, q, scale, (int)N, (int)K, acc, y, nw, st);
        case 3: return launch_dot4_g<3>(G, packed, beta, layout, q, scale, (int)N, (int)K, acc, y, nw, st);
        default: return launch_dot4_g<4>(G, packed, beta, layout, q, scale, (int)N, (int)K, acc, y, nw, st);
    }
}
