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
#include "bl_producer.h"

/* One decode product: everything a workgroup needs to know about it. */
struct bl_gemv_prob {
    const bl_v4i* packed;     /* N x K/64 units of 16 bytes                          */
    const int8_t* q;          /* [M][K] int8, or NULL when x is given               */
    bl_prod_dev prod;         /* fused paths: where the bf16 activations come from  */
    int fused;                /* 1: quantise prod's output on the fly; 0: use q     */
    const float* residual;    /* [M][N] or NULL: added to y in the epilogue         */
    const float* beta;
    const float* scale;       /* [M] input scale (q path; may be NULL if y == NULL) */
    const int32_t* rowsum;    /* [M] or NULL                                        */
    int32_t* acc;             /* [M][N] or NULL                                     */
    float* y;                 /* [M][N] or NULL                                     */
    int8_t* q_out;            /* fused path: optional copy of q, [M][K]             */
    float* scale_out;         /* fused path: optional [M]                           */
    int N, K, layout, block0; /* block0: first workgroup of this product            */
    int ksplit;               /* waves sharing one row group (1, 2 or 4)            */
    float fixed_scale;        /* fused path: > 0 replaces absmax/127 in the rescale */
};
#define BL_GEMV_MAX_GROUP 4
struct bl_gemv_group {
    bl_gemv_prob p[BL_GEMV_MAX_GROUP];
    int count;
};

/* LDS image of the activations.  For token m and 64-wide k chunk c, sixteen
 * dwords indexed [s][d]: the bytes that pair with bit-pair level s of packed
 * word d of the chunk.
 *   layout 1: level s of word d holds k = 16d+4s+{0..3}  -> natural dword 4d+s.
 *   layout 0: level s of word d holds k = 16d+{s,4+s,8+s,12+s} -> byte transpose.
 * put16 stores the sixteen int8 of k = 16*c16 .. 16*c16+15 (as four natural dwords). */
__device__ __forceinline__ void bl_put16(int* __restrict__ Qm, int c16, int layout, uint32_t a0, uint32_t a1,
                                         uint32_t a2, uint32_t a3) {
    if (layout == 0) bl_transpose4x4(a0, a1, a2, a3);
    int* dst = Qm + (c16 >> 2) * 16 + (c16 & 3);
    dst[0] = (int)a0;
    dst[4] = (int)a1;
    dst[8] = (int)a2;
    dst[12] = (int)a3;
}




/* One k chunk of the VALU path: the four bit-pair levels of the four packed
 * words against the staged activation dwords of one token.  Levels are
 * isolated by masks (one shift for the top level) and accumulated with the
 * factors 1, 4, 16, 16. */
__device__ __forceinline__ void bl_dot_chunk(const bl_v4i p, const bl_v4i* __restrict__ Qc, int* A) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const bl_v4i qs = Qc[s];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t w = (uint32_t)p[d];
            const uint32_t lv = s == 0 ? (w & 0x03030303u)
                              : s == 1 ? (w & 0x0C0C0C0Cu)
                              : s == 2 ? (w & 0x30303030u)
                                       : ((w >> 2) & 0x30303030u);
            A[s] = __builtin_amdgcn_sdot4((int)lv, qs[d], A[s], false);
        }
    }
}

/* Decode kernel, M <= 4 tokens, up to four independent products per launch.
 * Four waves per workgroup.  A row group is R = 64/G weight rows; `ksplit`
 * waves share a row group and split its k chunks between them (small N: more
 * workgroups; large N: ksplit = 1 and no cross-wave step at all).  Lane (r, g)
 * of k-part kp issues all of its L 128-bit weight loads (chunks (i*ksplit+kp)*G+g)
 * before anything else, so the HBM latency overlaps the activation staging; the
 * G lanes of a row are summed with DPP, k-parts through LDS.
 * Dynamic LDS: M*K bytes of staged activations + M ints + (M+4) floats + 64*M ints. */
template <int M, int G, int L>
__global__ __launch_bounds__(256) void bl_gemv_rows(const bl_gemv_group grp) {
    extern __shared__ int lds[];
    constexpr int R = 64 / G;
    int pi = 0;
#pragma unroll
    for (int i = 1; i < BL_GEMV_MAX_GROUP; ++i)
        if (i < grp.count && (int)blockIdx.x >= grp.p[i].block0) pi = i;
    const bl_gemv_prob& P = grp.p[pi];
    const int N = P.N, K = P.K, nchunks = K / 64, ksplit = P.ksplit;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane / G, g = lane % G;
    const int rg = w / ksplit, kp = w - rg * ksplit;          /* row group in block, k part */
    const int rows_per_block = (4 / ksplit) * R;
    const int n = ((int)blockIdx.x - P.block0) * rows_per_block + rg * R + r;
    const bool row_ok = n < N;

    /* activation loads first, so that staging needs to wait for them only */
    const int groups = K / 16;
    uint4 xv[4];
    bl_v4i qv = {0, 0, 0, 0};
    const bool pre_bf16 = P.fused && P.prod.kind == BL_PROD_BF16;
    const bool first_block = blockIdx.x == (unsigned)P.block0;
    if (pre_bf16) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int u = tid + j * 256;
            if (u < groups) {
                xv[2 * j] = ((const uint4*)P.prod.in0)[2 * u];
                xv[2 * j + 1] = ((const uint4*)P.prod.in0)[2 * u + 1];
            }
        }
    } else if (!P.fused && tid < M * groups) {
        qv = *(const bl_v4i*)(P.q + (int64_t)(tid / groups) * K + (int64_t)(tid % groups) * 16);
    }

    bl_v4i p[L];
    {
        const bl_v4i* wrow = P.packed + (int64_t)(row_ok ? n : 0) * nchunks;
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int chunk = (i * ksplit + kp) * G + g;
            p[i] = bl_v4i{0, 0, 0, 0};
            if (row_ok && chunk < nchunks) p[i] = __builtin_nontemporal_load(wrow + chunk);
        }
    }

    int* Q = lds;                       /* M*K/4 dwords                      */
    int* sq = Q + M * (K / 4);          /* M row sums                        */
    float* fs = (float*)(sq + M);       /* M scales, then 4 per-wave scratch */
    int* red = (int*)(fs + M + 4);      /* 4 waves * R * M partial sums      */
    if (P.fused) {
        if (tid < M) sq[tid] = 0;                  /* ordered before the atomics by the absmax barrier */
        /* fused producer: absmax + int8 quantisation of the bf16 row, per token.
         * Each thread keeps its (at most two) 16-element groups in registers. */
#pragma unroll 1
        for (int m = 0; m < M; ++m) {
            float mx = 0.0f;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = tid + j * 256;
                if (u < groups) {
                    if (m > 0 || !pre_bf16) bl_produce16(P.prod, m, u, K, first_block, xv[2 * j], xv[2 * j + 1]);
                    mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(xv[2 * j]), bl_absmax8_bf16(xv[2 * j + 1])));
                }
            }
            for (int u = tid + 512; u < groups; u += 256) {
                uint4 lo, hi;
                bl_produce16(P.prod, m, u, K, false, lo, hi);
                mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(lo), bl_absmax8_bf16(hi)));
            }
            mx = bl_wave_max(mx);
            if (lane == 0) fs[M + w] = mx;
            __syncthreads();
            const float gamma = fmaxf(fmaxf(fs[M], fs[M + 1]), fmaxf(fs[M + 2], fs[M + 3]));
            const float gg = fmaxf(gamma, 1e-5f);
            const float inv = bl_div_rn(127.0f, gg);
            const bool emit = P.q_out && first_block;
            int part = 0;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = tid + j * 256;
                if (u < groups) {
                    uint32_t a0, a1, a2, a3;
                    bl_quant8_words(xv[2 * j], inv, a0, a1);
                    bl_quant8_words(xv[2 * j + 1], inv, a2, a3);
                    part += bl_sum16(a0, a1, a2, a3);
                    if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                    bl_put16(Q + m * (K / 4), u, P.layout, a0, a1, a2, a3);
                }
            }
            for (int u = tid + 512; u < groups; u += 256) {
                uint32_t a0, a1, a2, a3;
                uint4 lo, hi;
                bl_produce16(P.prod, m, u, K, first_block, lo, hi);
                bl_quant8_words(lo, inv, a0, a1);
                bl_quant8_words(hi, inv, a2, a3);
                part += bl_sum16(a0, a1, a2, a3);
                if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                bl_put16(Q + m * (K / 4), u, P.layout, a0, a1, a2, a3);
            }
            part = bl_wave_sum(part);
            if (lane == 0) atomicAdd(&sq[m], part);   /* four LDS atomics per token */
            if (tid == 0) {
                const float sc = bl_div_rn(gg, 127.0f);
                fs[m] = P.fixed_scale > 0.0f ? P.fixed_scale : sc;
                if (P.scale_out && first_block) P.scale_out[m] = sc;
            }
            __syncthreads();                       /* Q, sq[m], fs[m] complete; fs[M..] reusable */
        }
    } else {
        const bool need_sum = P.rowsum == nullptr;
        if (tid < M) {
            sq[tid] = need_sum ? 0 : P.rowsum[tid];
            fs[tid] = P.scale ? P.scale[tid] : 0.0f;
        }
        if (need_sum) __syncthreads();
        for (int u = tid; u < M * groups; u += 256) {
            const int m = u / groups, c16 = u - m * groups;
            bl_v4i v = qv;
            if (u >= 256) v = *(const bl_v4i*)(P.q + (int64_t)m * K + (int64_t)c16 * 16);
            if (need_sum) atomicAdd(&sq[m], bl_sum16((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]));
            bl_put16(Q + m * (K / 4), c16, P.layout, (uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]);
        }
        __syncthreads();
    }

    int A[M][4];
#pragma unroll
    for (int m = 0; m < M; ++m) A[m][0] = A[m][1] = A[m][2] = A[m][3] = 0;
#pragma unroll
    for (int i = 0; i < L; ++i) {
        const int chunk = (i * ksplit + kp) * G + g;
        if (chunk < nchunks) {
#pragma unroll
            for (int m = 0; m < M; ++m)
                bl_dot_chunk(p[i], (const bl_v4i*)(Q + (m * nchunks + chunk) * 16), A[m]);
        }
    }
    const float bt = *P.beta;
    int v[M];
#pragma unroll
    for (int m = 0; m < M; ++m)
        v[m] = bl_group_sum<G>(A[m][0] + (A[m][1] >> 2) + ((A[m][2] + A[m][3]) >> 4));
    /* Lanes 0..R-1 of the first wave of a row group write rows 0..R-1: one
     * contiguous R*4-byte store per token instead of R scattered dwords. */
    int o[M];
    if (ksplit > 1) {
        if (g == 0) {
#pragma unroll
            for (int m = 0; m < M; ++m) red[(w * R + r) * M + m] = v[m];
        }
        __syncthreads();
        if (kp == 0 && lane < R) {
#pragma unroll
            for (int m = 0; m < M; ++m) {
                o[m] = 0;
                for (int j = 0; j < ksplit; ++j) o[m] += red[((w + j) * R + lane) * M + m];
            }
        }
    } else {
#pragma unroll
        for (int m = 0; m < M; ++m) o[m] = __shfl(v[m], (lane & (R - 1)) * G);
    }
    const int n_out = ((int)blockIdx.x - P.block0) * rows_per_block + rg * R + lane;
    if (kp == 0 && lane < R && n_out < N) {
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int val = o[m] - sq[m];
            if (P.acc) P.acc[(int64_t)m * N + n_out] = val;
            if (P.y) {
                const float t = (float)val * (bt * fs[m]);
                P.y[(int64_t)m * N + n_out] = P.residual ? P.residual[(int64_t)m * N + n_out] + t : t;
            }
        }
    }
}

#define BL_MMA_PAD 16   /* bytes added to each staged activation row (LDS bank spread) */

/* Matrix-core decode kernel, M <= 16*MT tokens, up to four products per launch.
 * Same work split as bl_gemv_rows with G = 4: lane (c, kg) owns weight row c of
 * a 16-row group and k chunks (i*ksplit+kp)*4+kg.  Each 16-byte weight load
 * feeds four v_mfma_i32_16x16x64_i8, one per bit-pair level s: the B operand is
 * the lane's four packed words masked to level s (no shift except the top
 * level), the A operand the activation bytes of token l%16 that pair with that
 * level, read from the LDS image [chunk][s][d] by the lanes of real tokens only.
 * The four levels accumulate separately with factors 1, 4, 16, 16 (four
 * independent MFMA chains) and are recombined once with exact shifts.  The k
 * reduction happens inside the matrix core: no cross-lane step.  sum_k q comes
 * from a fifth chain with an all-ones B operand when no rowsum was given.
 * The activation loads are issued before the weight loads so that staging can
 * proceed while the weights are still in flight.
 * Dynamic LDS: M*(K+16) bytes + (MT*2*4*256 + 4 + 64) ints. */
template <int L, int MT, bool NEED_SUM>
__global__ __launch_bounds__(256) void bl_gemv_mma(const bl_gemv_group grp, const int M) {
    extern __shared__ int lds[];
    int pi = 0;
#pragma unroll
    for (int i = 1; i < BL_GEMV_MAX_GROUP; ++i)
        if (i < grp.count && (int)blockIdx.x >= grp.p[i].block0) pi = i;
    const bl_gemv_prob& P = grp.p[pi];
    const int N = P.N, K = P.K, nchunks = K / 64, ksplit = P.ksplit;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int c = lane & 15, kg = lane >> 4;
    const int rg = w / ksplit, kp = w - rg * ksplit;
    const int rows_per_block = (4 / ksplit) * 16;
    const int n = ((int)blockIdx.x - P.block0) * rows_per_block + rg * 16 + c;
    const bool row_ok = n < N;
    const int groups = K / 16;
    const int qstride = K + BL_MMA_PAD;                 /* bytes per staged token row */
    uint8_t* Q = (uint8_t*)lds;
    int* red = (int*)(Q + M * qstride);                 /* C and Cs of 4 waves, MT tiles */
    float* fs = (float*)(red + MT * 4 * 256 * 2);       /* 4 wave maxima                 */
    float* fscale = fs + 4;                             /* M scales (fused path)         */

    /* 1. activation loads first (token 0 of the fused path, or the first q groups) */
    uint4 xv[4];
    bl_v4i qv = {0, 0, 0, 0};
    const bool pre_bf16 = P.fused && P.prod.kind == BL_PROD_BF16;
    const bool first_block = blockIdx.x == (unsigned)P.block0;
    if (pre_bf16) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int u = tid + j * 256;
            if (u < groups) {
                xv[2 * j] = ((const uint4*)P.prod.in0)[2 * u];
                xv[2 * j + 1] = ((const uint4*)P.prod.in0)[2 * u + 1];
            }
        }
    } else if (!P.fused && tid < M * groups) {
        qv = *(const bl_v4i*)(P.q + (int64_t)(tid / groups) * K + (int64_t)(tid % groups) * 16);
    }

    /* 2. every weight load of this lane */
    bl_v4i p[L];
    {
        const bl_v4i* wrow = P.packed + (int64_t)(row_ok ? n : 0) * nchunks;
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int chunk = (i * ksplit + kp) * 4 + kg;
            p[i] = bl_v4i{0, 0, 0, 0};
            if (row_ok && chunk < nchunks) p[i] = __builtin_nontemporal_load(wrow + chunk);
        }
    }

    /* 3. stage the activations */
    if (P.fused) {
#pragma unroll 1
        for (int m = 0; m < M; ++m) {
            float mx = 0.0f;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = tid + j * 256;
                if (u < groups) {
                    if (m > 0 || !pre_bf16) bl_produce16(P.prod, m, u, K, first_block, xv[2 * j], xv[2 * j + 1]);
                    mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(xv[2 * j]), bl_absmax8_bf16(xv[2 * j + 1])));
                }
            }
            for (int u = tid + 512; u < groups; u += 256) {
                uint4 lo, hi;
                bl_produce16(P.prod, m, u, K, false, lo, hi);
                mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(lo), bl_absmax8_bf16(hi)));
            }
            mx = bl_wave_max(mx);
            if (m > 0) __syncthreads();                 /* previous token's fs[] readers are done */
            if (lane == 0) fs[w] = mx;
            __syncthreads();
            const float gamma = fmaxf(fmaxf(fs[0], fs[1]), fmaxf(fs[2], fs[3]));
            const float gg = fmaxf(gamma, 1e-5f);
            const float inv = bl_div_rn(127.0f, gg);
            const bool emit = P.q_out && first_block;
            int* Qm = (int*)(Q + m * qstride);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = tid + j * 256;
                if (u < groups) {
                    uint32_t a0, a1, a2, a3;
                    bl_quant8_words(xv[2 * j], inv, a0, a1);
                    bl_quant8_words(xv[2 * j + 1], inv, a2, a3);
                    if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                    bl_put16(Qm, u, P.layout, a0, a1, a2, a3);
                }
            }
            for (int u = tid + 512; u < groups; u += 256) {
                uint32_t a0, a1, a2, a3;
                uint4 lo, hi;
                bl_produce16(P.prod, m, u, K, first_block, lo, hi);
                bl_quant8_words(lo, inv, a0, a1);
                bl_quant8_words(hi, inv, a2, a3);
                if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                bl_put16(Qm, u, P.layout, a0, a1, a2, a3);
            }
            if (tid == 0) {
                const float sc = bl_div_rn(gg, 127.0f);
                fscale[m] = P.fixed_scale > 0.0f ? P.fixed_scale : sc;
                if (P.scale_out && first_block) P.scale_out[m] = sc;
            }
        }
    } else {
        if (tid < M * groups)
            bl_put16((int*)(Q + (tid / groups) * qstride), tid % groups, P.layout, (uint32_t)qv[0], (uint32_t)qv[1],
                     (uint32_t)qv[2], (uint32_t)qv[3]);
        for (int u = tid + 256; u < M * groups; u += 256) {
            const int m = u / groups, c16 = u - m * groups;
            const uint4 v = *(const uint4*)(P.q + (int64_t)m * K + (int64_t)c16 * 16);
            bl_put16((int*)(Q + m * qstride), c16, P.layout, v.x, v.y, v.z, v.w);
        }
    }
    __syncthreads();

    /* 4. products: four levels, four accumulators per token tile */
    constexpr bool need_sum = NEED_SUM;   /* the launcher checked: no product of the group has a rowsum */
    const bl_v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    bl_v4i C[MT][4], Cs[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) C[t][0] = C[t][1] = C[t][2] = C[t][3] = Cs[t] = bl_v4i{0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < L; ++i) {
        const int chunk = (i * ksplit + kp) * 4 + kg;
        const bool cv = chunk < nchunks;
        if ((i * ksplit + kp) * 4 < nchunks) {          /* wave-uniform: some lane has work */
            const bl_v4i pw = p[i];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                bl_v4i b;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t wd = (uint32_t)pw[d];
                    b[d] = (int)(s == 0 ? (wd & 0x03030303u)
                               : s == 1 ? (wd & 0x0C0C0C0Cu)
                               : s == 2 ? (wd & 0x30303030u)
                                        : ((wd >> 2) & 0x30303030u));
                }
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const int tok = t * 16 + c;
                    bl_v4i a = {0, 0, 0, 0};
                    if (cv && tok < M) a = *(const bl_v4i*)(Q + tok * qstride + chunk * 64 + s * 16);
                    C[t][s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, C[t][s], 0, 0, 0);
                    if (need_sum) Cs[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, ones, Cs[t], 0, 0, 0);
                }
            }
        }
    }
    bl_v4i D[MT];
    bl_mfma_fence();
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            D[t][v] = C[t][0][v] + (C[t][1][v] >> 2) + ((C[t][2][v] + C[t][3][v]) >> 4) - Cs[t][v];

    if (ksplit > 1) {
#pragma unroll
        for (int t = 0; t < MT; ++t) *(bl_v4i*)(red + ((t * 4 + w) * 64 + lane) * 4) = D[t];
        __syncthreads();
        if (kp == 0) {
            for (int j = 1; j < ksplit; ++j)
#pragma unroll
                for (int t = 0; t < MT; ++t) D[t] += *(const bl_v4i*)(red + ((t * 4 + w + j) * 64 + lane) * 4);
        }
    }
    if (kp == 0 && row_ok) {
        const float bt = *P.beta;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int tok = t * 16 + kg * 4 + v;
                if (tok < M) {
                    const int val = D[t][v] - (need_sum ? 0 : P.rowsum[tok]);
                    if (P.acc) P.acc[(int64_t)tok * N + n] = val;
                    if (P.y) {
                        const float sc = P.fused ? fscale[tok] : P.scale[tok];
                        const float t = (float)val * (bt * sc);
                        P.y[(int64_t)tok * N + n] = P.residual ? P.residual[(int64_t)tok * N + n] + t : t;
                    }
                }
            }
    }
}

static int bl_env_int(const char* name, int dflt) {
    const char* e = getenv(name);
    return e && *e ? atoi(e) : dflt;
}

template <int M, int G, int L>
static bl_status launch_rows(const bl_gemv_group& grp, int blocks, int maxK, hipStream_t st) {
    const size_t lds = (size_t)M * maxK + (size_t)M * 4 + (size_t)(M + 4) * 4 + (size_t)64 * M * 4;
    if (lds > 64 * 1024) return BL_ERR_SHAPE;
    bl_gemv_rows<M, G, L><<<blocks, 256, lds, st>>>(grp);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

template <int M, int G>
static bl_status launch_rows_l(int L, const bl_gemv_group& grp, int blocks, int maxK, hipStream_t st) {
    if (L <= 2) return launch_rows<M, G, 2>(grp, blocks, maxK, st);
    if (L <= 4) return launch_rows<M, G, 4>(grp, blocks, maxK, st);
    if (L <= 8) return launch_rows<M, G, 8>(grp, blocks, maxK, st);
    if (L <= 16) return launch_rows<M, G, 16>(grp, blocks, maxK, st);
    return launch_rows<M, G, 32>(grp, blocks, maxK, st);
}

template <int L, int MT>
static bl_status launch_mma(const bl_gemv_group& grp, int M, int blocks, int maxK, hipStream_t st) {
    const size_t lds = (size_t)M * (maxK + BL_MMA_PAD) + (size_t)(MT * 4 * 256 * 2 + 4 + 64) * 4;
    bool have_sums = true;   /* every product brings its own row sums */
    for (int i = 0; i < grp.count; ++i)
        if (grp.p[i].fused || !grp.p[i].rowsum) have_sums = false;
    auto kern = have_sums ? bl_gemv_mma<L, MT, false> : bl_gemv_mma<L, MT, true>;
    if (lds > 160 * 1024) return BL_ERR_SHAPE;
    if (lds > 64 * 1024) {
        static bool done[2] = {false, false};
        if (!done[have_sums]) {
            if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) !=
                hipSuccess)
                return BL_ERR_HIP;
            done[have_sums] = true;
        }
    }
    kern<<<blocks, 256, lds, st>>>(grp, M);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

template <int MT>
static bl_status launch_mma_l(int L, const bl_gemv_group& grp, int M, int blocks, int maxK, hipStream_t st) {
    if (L <= 2) return launch_mma<2, MT>(grp, M, blocks, maxK, st);
    if (L <= 4) return launch_mma<4, MT>(grp, M, blocks, maxK, st);
    if (L <= 8) return launch_mma<8, MT>(grp, M, blocks, maxK, st);
    if (L <= 16) return launch_mma<16, MT>(grp, M, blocks, maxK, st);
    return launch_mma<32, MT>(grp, M, blocks, maxK, st);
}

/* Lays the products of a group out over workgroups and launches them.  All
 * products of a group share M.  k is split over the waves of a workgroup when
 * a product alone would give fewer than about 150 workgroups.
 * Path: the VALU dot4 + DPP kernel for M <= 4 (measured faster there), the
 * matrix-core kernel above that; BL_GEMV_PATH=mma forces the latter.  Returns BL_ERR_SHAPE if a K is too long for the
 * register-resident row scheme (the caller then uses the prefill kernel). */
bl_status bl_gemv_launch_group(bl_gemv_group& grp, int M, hipStream_t st) {
    const char* path_env = getenv("BL_GEMV_PATH");
    const bool dot4 = M <= 4 && !(path_env && path_env[0] == 'm');
    int G = dot4 ? bl_env_int("BL_GEMV_G", 8) : 4;
    if (G != 4 && G != 8) G = 8;
    const int force_split = bl_env_int("BL_GEMV_KSPLIT", 0);
    const int want_blocks = bl_env_int("BL_GEMV_BLOCKS", 150);   /* measured best of 60..700 */
    const int R = 64 / G;
    int blocks = 0, maxK = 0, L = 0;
    for (int i = 0; i < grp.count; ++i) {
        bl_gemv_prob& P = grp.p[i];
        int ks = 1;
        while (ks < 4 && (P.N + (4 / ks) * R - 1) / ((4 / ks) * R) < want_blocks) ks *= 2;
        if (force_split == 1 || force_split == 2 || force_split == 4) ks = force_split;
        P.ksplit = ks;
        P.block0 = blocks;
        const int rows_per_block = (4 / ks) * R;
        blocks += (P.N + rows_per_block - 1) / rows_per_block;
        if (P.K > maxK) maxK = P.K;
        const int l = (P.K / 64 + G * ks - 1) / (G * ks);
        if (l > L) L = l;
    }
    if (L > 32) return BL_ERR_SHAPE;
    if (!dot4) {
        if (M <= 16) return launch_mma_l<1>(L, grp, M, blocks, maxK, st);
        if (M <= 32) return launch_mma_l<2>(L, grp, M, blocks, maxK, st);
        return launch_mma_l<4>(L, grp, M, blocks, maxK, st);
    }
    switch (M * 10 + G) {
        case 14: return launch_rows_l<1, 4>(L, grp, blocks, maxK, st);
        case 18: return launch_rows_l<1, 8>(L, grp, blocks, maxK, st);
        case 24: return launch_rows_l<2, 4>(L, grp, blocks, maxK, st);
        case 28: return launch_rows_l<2, 8>(L, grp, blocks, maxK, st);
        case 34: return launch_rows_l<3, 4>(L, grp, blocks, maxK, st);
        case 38: return launch_rows_l<3, 8>(L, grp, blocks, maxK, st);
        case 44: return launch_rows_l<4, 4>(L, grp, blocks, maxK, st);
        default: return launch_rows_l<4, 8>(L, grp, blocks, maxK, st);
    }
}

bl_status bl_gemm_dispatch(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                           const float* scale, const int32_t* rowsum, int64_t M, int64_t N, int64_t K,
                           const float* residual, int32_t* acc, float* y, void* workspace, hipStream_t st);

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
    if (K > 8192 || M * (K + BL_MMA_PAD) > 96 * 1024)
        return bl_gemm_dispatch(packed, beta, layout, q, scale, rowsum, M, N, K, nullptr, acc, y, workspace, st);

    bl_gemv_group grp;
    grp.count = 1;
    bl_gemv_prob& P0 = grp.p[0];
    P0 = bl_gemv_prob{};
    P0.packed = (const bl_v4i*)packed; P0.q = q; P0.beta = beta; P0.scale = scale; P0.rowsum = rowsum;
    P0.acc = acc; P0.y = y; P0.N = (int)N; P0.K = (int)K; P0.layout = layout; P0.ksplit = 1;
    return bl_gemv_launch_group(grp, (int)M, st);
}

static bl_status check_decode_desc(const bl_decode_desc& d, int64_t M, int layout) {
    if (!d.packed || !d.beta) return BL_ERR_NULL;
    const bool fused = d.X || d.prod.in0;
    if (!fused && !d.q) return BL_ERR_NULL;
    if (!d.acc && !d.y) return BL_ERR_NULL;
    if (!fused && d.y && !d.scale) return BL_ERR_NULL;
    if (M < 1 || M > 16 || !bl_shape_ok(d.N, d.K) || d.K > 8192 || M * (d.K + BL_MMA_PAD) > 96 * 1024)
        return BL_ERR_SHAPE;
    if (layout != BL_LAYOUT_ROWMAJOR && layout != BL_LAYOUT_K16) return BL_ERR_LAYOUT;
    if (!bl_aligned(d.packed, 16) || !bl_aligned(d.X, 16) || !bl_aligned(d.q, 16) || !bl_aligned(d.q_out, 16) ||
        !bl_aligned(d.acc, 4) || !bl_aligned(d.y, 4) || !bl_aligned(d.scale, 4) || !bl_aligned(d.beta, 4) ||
        !bl_aligned(d.rowsum, 4) || !bl_aligned(d.scale_out, 4) || !bl_aligned(d.residual, 4))
        return BL_ERR_ALIGN;
    return BL_OK;
}

extern "C" bl_status bl_bitlinear_decode_group(const bl_decode_desc* descs, int count, int layout, int64_t M,
                                               bl_stream s) {
    if (!descs) return BL_ERR_NULL;
    if (count < 1 || count > BL_GEMV_MAX_GROUP) return BL_ERR_SHAPE;
    bl_gemv_group grp;
    grp.count = count;
    for (int i = 0; i < count; ++i) {
        const bl_decode_desc& d = descs[i];
        const bl_status st = check_decode_desc(d, M, layout);
        if (st != BL_OK) return st;
        bl_gemv_prob& P = grp.p[i];
        P = bl_gemv_prob{};
        P.fused = (d.X || d.prod.in0) ? 1 : 0;
        if (P.fused && !bl_make_prod(d.prod, d.X, d.K, &P.prod)) return BL_ERR_VALUE;
        P.packed = (const bl_v4i*)d.packed; P.q = P.fused ? nullptr : d.q; P.beta = d.beta; P.scale = d.scale;
        P.rowsum = d.rowsum; P.acc = d.acc; P.y = d.y; P.q_out = d.q_out; P.scale_out = d.scale_out;
        P.N = (int)d.N; P.K = (int)d.K; P.layout = layout; P.ksplit = 1; P.fixed_scale = d.fixed_scale;
        P.residual = d.residual;
    }
    return bl_gemv_launch_group(grp, (int)M, (hipStream_t)s);
}

extern "C" bl_status bl_bitlinear_decode(const uint8_t* packed, const float* beta, int layout, const uint16_t* X,
                                         int64_t M, int64_t N, int64_t K, int32_t* acc, float* y, int8_t* q_out,
                                         float* scale_out, bl_stream s) {
    if (!X) return BL_ERR_NULL;
    bl_decode_desc d = {};
    d.packed = packed; d.beta = beta; d.X = X; d.N = N; d.K = K; d.acc = acc; d.y = y;
    d.q_out = q_out; d.scale_out = scale_out;
    return bl_bitlinear_decode_group(&d, 1, layout, M, s);
}
