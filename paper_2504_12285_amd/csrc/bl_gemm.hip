/* Prefill-side W1.58A8 product (Section 5.1 of the BitNet b1.58 2B4T report):
 * a dense int8 contraction on the CDNA4 matrix cores.  Packed 2-bit weight
 * tiles go HBM -> LDS still packed (a quarter of the int8 bytes), each wave
 * expands the words it needs to int8 in registers with shift+mask right before
 * v_mfma_i32_32x32x32_i8, and the activations stream through LDS as int8.
 * Codes c = Wt + 1 are contracted as they are; the epilogue subtracts
 * rowsum[m] = sum_k q[m][k] (exact int32 identity), then rescales.
 */
#include "bl_device.h"
#include "bl_host.h"

#define GEMM_THREADS 256
#define GEMM_BK 64
#define A_STRIDE 80   /* bytes per activation row in LDS: 64 + 16 pad */
#define W_STRIDE 5    /* dwords per packed weight row in LDS: 4 + 1 pad */

template <int BM, int BN, int LAYOUT>
__global__ __launch_bounds__(GEMM_THREADS) void bl_gemm_mfma(const uint8_t* __restrict__ packed,
                                                              const int8_t* __restrict__ q,
                                                              const int32_t* __restrict__ rowsum,
                                                              const float* __restrict__ beta,
                                                              const float* __restrict__ scale, int M, int N, int K,
                                                              int32_t* __restrict__ acc, float* __restrict__ y) {
    constexpr int WM = BM / 2, WN = BN / 2, MI = WM / 32, NI = WN / 32;
    constexpr int A_UNITS = BM * 4 / GEMM_THREADS;  /* 16-byte units per thread */
    __shared__ __attribute__((aligned(16))) uint8_t As[BM * A_STRIDE];
    __shared__ uint32_t Ws[BN * W_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int l32 = lane & 31, h = lane >> 5;
    const int kb = K / 4;  /* packed bytes per weight row */

    bl_v16i C[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) C[mi][ni][v] = 0;

    /* global -> register staging */
    uint4 areg[A_UNITS];
    uint4 wreg = make_uint4(0, 0, 0, 0);
    const uint8_t* aptr[A_UNITS];
#pragma unroll
    for (int i = 0; i < A_UNITS; ++i) {
        const int u = tid + i * GEMM_THREADS, row = u >> 2, c = u & 3;
        int m = m0 + row;
        if (m >= M) m = M - 1;
        aptr[i] = (const uint8_t*)q + (int64_t)m * K + c * 16;
    }
    int wn = n0 + tid;
    if (wn >= N) wn = N - 1;
    const uint8_t* wptr = packed + (int64_t)wn * kb;
    const bool wload = tid < BN;

    auto load_tiles = [&](int kk) {
#pragma unroll
        for (int i = 0; i < A_UNITS; ++i) areg[i] = *(const uint4*)(aptr[i] + (int64_t)kk * GEMM_BK);
        if (wload) wreg = *(const uint4*)(wptr + (int64_t)kk * 16);
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int i = 0; i < A_UNITS; ++i) {
            const int u = tid + i * GEMM_THREADS, row = u >> 2, c = u & 3;
            uint32_t a0 = areg[i].x, a1 = areg[i].y, a2 = areg[i].z, a3 = areg[i].w;
            if (LAYOUT == 0) bl_transpose4x4(a0, a1, a2, a3);
            *(uint4*)(As + row * A_STRIDE + c * 16) = make_uint4(a0, a1, a2, a3);
        }
        if (wload) {
            uint32_t* d = Ws + tid * W_STRIDE;
            d[0] = wreg.x; d[1] = wreg.y; d[2] = wreg.z; d[3] = wreg.w;
        }
    };

    const int steps = K / GEMM_BK;
    load_tiles(0);
    store_tiles();
    __syncthreads();
    for (int kk = 0; kk < steps; ++kk) {
        if (kk + 1 < steps) load_tiles(kk + 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bl_v4i a[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                a[mi] = *(const bl_v4i*)(As + (wm0 + mi * 32 + l32) * A_STRIDE + ks * 32 + h * 16);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const uint32_t p = Ws[(wn0 + ni * 32 + l32) * W_STRIDE + ks * 2 + h];
                bl_v4i b;
                b[0] = (int)(p & 0x03030303u);
                b[1] = (int)((p >> 2) & 0x03030303u);
                b[2] = (int)((p >> 4) & 0x03030303u);
                b[3] = (int)((p >> 6) & 0x03030303u);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    C[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], b, C[mi][ni], 0, 0, 0);
            }
        }
        __syncthreads();
        if (kk + 1 < steps) store_tiles();
        __syncthreads();
    }

    const float bt = *beta;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + wm0 + mi * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
            if (m < M) {
                const int rs = rowsum[m];
                const float c = y ? bt * scale[m] : 0.0f;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const int n = n0 + wn0 + ni * 32 + l32;
                    if (n < N) {
                        const int val = C[mi][ni][v] - rs;
                        if (acc) acc[(int64_t)m * N + n] = val;
                        if (y) y[(int64_t)m * N + n] = (float)val * c;
                    }
                }
            }
        }
}

/* rowsum[m] = sum_k q[m][k]; one wave per row. */
__global__ __launch_bounds__(256) void bl_rowsum_kernel(const int8_t* __restrict__ q, int M, int K,
                                                         int32_t* __restrict__ rowsum) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const uint4* row = (const uint4*)(q + (int64_t)m * K);
    int s = 0;
    for (int i = lane; i < K / 16; i += 64) {
        const uint4 v = row[i];
        s = __builtin_amdgcn_sdot4((int)v.x, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4((int)v.y, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4((int)v.z, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4((int)v.w, 0x01010101, s, false);
    }
    s = bl_wave_sum(s);
    if (lane == 0) rowsum[m] = s;
}

/* Arguments already validated by the public entry points. */
bl_status bl_gemm_dispatch(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                           const float* scale, const int32_t* rowsum, int64_t M, int64_t N, int64_t K,
                           int32_t* acc, float* y, void* workspace, hipStream_t st) {
    if (!rowsum) {
        if (!workspace) return BL_ERR_WORKSPACE;
        if (!bl_aligned(workspace, 4)) return BL_ERR_ALIGN;
        int32_t* rs = (int32_t*)workspace;
        bl_rowsum_kernel<<<(unsigned)((M + 3) / 4), 256, 0, st>>>(q, (int)M, (int)K, rs);
        rowsum = rs;
    }
    constexpr int BM = 128, BN = 128;
    dim3 grid((unsigned)((N + BN - 1) / BN), (unsigned)((M + BM - 1) / BM));
    if (layout == 0)
        bl_gemm_mfma<BM, BN, 0><<<grid, GEMM_THREADS, 0, st>>>(packed, q, rowsum, beta, scale, (int)M, (int)N,
                                                               (int)K, acc, y);
    else
        bl_gemm_mfma<BM, BN, 1><<<grid, GEMM_THREADS, 0, st>>>(packed, q, rowsum, beta, scale, (int)M, (int)N,
                                                               (int)K, acc, y);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

extern "C" bl_status bl_gemm_w158a8(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                                    const float* scale, const int32_t* rowsum, int64_t M, int64_t N, int64_t K,
                                    int32_t* acc, float* y, void* workspace, bl_stream s) {
    if (!packed || !beta || !q) return BL_ERR_NULL;
    if (!acc && !y) return BL_ERR_NULL;
    if (y && !scale) return BL_ERR_NULL;
    if (M < 1 || M > BL_MAX_DIM || !bl_shape_ok(N, K)) return BL_ERR_SHAPE;
    if (layout != BL_LAYOUT_ROWMAJOR && layout != BL_LAYOUT_K16) return BL_ERR_LAYOUT;
    if (!bl_aligned(packed, 16) || !bl_aligned(q, 16) || !bl_aligned(acc, 4) || !bl_aligned(y, 4) ||
        !bl_aligned(scale, 4) || !bl_aligned(beta, 4) || !bl_aligned(rowsum, 4))
        return BL_ERR_ALIGN;
    return bl_gemm_dispatch(packed, beta, layout, q, scale, rowsum, M, N, K, acc, y, workspace, (hipStream_t)s);
}
