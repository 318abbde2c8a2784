/* Weight quantisation (absmean -> ternary, Section 2 of the BitNet b1.58 2B4T
 * report) and 2-bit packing (Section 5.1), plus the inverse for round trips.
 * Offline step: bandwidth-trivial, but every bit must match the definition in
 * bitlinear.h. */
#include "bl_device.h"
#include "bl_host.h"

#define PACK_THREADS 256

/* Partial sums of |W| in fp64: block b sums a contiguous span of float4s in a
 * fixed order (thread-strided, then a fixed LDS tree). */
__global__ __launch_bounds__(PACK_THREADS) void bl_abs_sum_partial(const float4* __restrict__ W,
                                                                    int64_t n4, double* __restrict__ partial) {
    __shared__ double red[PACK_THREADS];
    const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x;
    const int64_t hi = lo + per < n4 ? lo + per : n4;
    double s = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += PACK_THREADS) {
        const float4 v = W[i];
        s += (double)fabsf(v.x);
        s += (double)fabsf(v.y);
        s += (double)fabsf(v.z);
        s += (double)fabsf(v.w);
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = PACK_THREADS / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

/* Fixed-order sum of the partials, mean in fp64, one rounding to fp32. */
__global__ __launch_bounds__(PACK_THREADS) void bl_abs_sum_final(const double* __restrict__ partial, int np,
                                                                  double count, float* __restrict__ beta) {
    __shared__ double red[PACK_THREADS];
    double s = 0.0;
    for (int i = threadIdx.x; i < np; i += PACK_THREADS) s += partial[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = PACK_THREADS / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *beta = (float)(red[0] / count);
}

/* Bit position of weight i (0..15) inside its 32-bit word. */
template <int LAYOUT>
__device__ __forceinline__ int bl_bitpos(int i) {
    return LAYOUT == 0 ? 2 * i : 8 * (i & 3) + 2 * (i >> 2);
}

template <int LAYOUT>
__device__ __forceinline__ uint32_t bl_code_word(const int* c) {
    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) w |= (uint32_t)c[i] << bl_bitpos<LAYOUT>(i);
    return w;
}

/* One thread = 16 consecutive k of one row = one packed word. */
template <int LAYOUT>
__global__ __launch_bounds__(PACK_THREADS) void bl_ternarize_pack(const float4* __restrict__ W,
                                                                   const float* __restrict__ beta, int64_t words,
                                                                   uint32_t* __restrict__ packed) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const float d = *beta + 1e-5f;
    int c[16];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float4 v = W[g * 4 + j];
        const float f[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float t = rintf(bl_div_rn(f[e], d));
            t = fminf(fmaxf(t, -1.0f), 1.0f);
            c[4 * j + e] = (int)t + 1;
        }
    }
    packed[g] = bl_code_word<LAYOUT>(c);
}

/* Same packing for weights that are already ternary int8. */
template <int LAYOUT>
__global__ __launch_bounds__(PACK_THREADS) void bl_pack_int8(const bl_v4i* __restrict__ Wt, int64_t words,
                                                              uint32_t* __restrict__ packed) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const bl_v4i v = Wt[g];
    int c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int b = (int)(int8_t)((uint32_t)v[i >> 2] >> (8 * (i & 3)));
        c[i] = (b < -1 ? -1 : (b > 1 ? 1 : b)) + 1;
    }
    packed[g] = bl_code_word<LAYOUT>(c);
}

template <int LAYOUT>
__global__ __launch_bounds__(PACK_THREADS) void bl_unpack_kernel(const uint32_t* __restrict__ packed, int64_t words,
                                                                  bl_v4i* __restrict__ Wt, int32_t* __restrict__ bad) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const uint32_t w = packed[g];
    bl_v4i out = {0, 0, 0, 0};
    int nbad = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = (int)((w >> bl_bitpos<LAYOUT>(i)) & 3u);
        nbad += (c == 3);
        out[i >> 2] |= (int)(((uint32_t)(c - 1) & 0xFFu) << (8 * (i & 3)));
    }
    Wt[g] = out;
    if (nbad) atomicAdd(bad, nbad);
}

/* ---- shapes with a ragged K (not a multiple of 64) or N (not a multiple of 4) ------------------
 * Element-wise versions of the kernels above: the packed matrix has Np rows of Kp weights and
 * every field outside the N x K matrix holds code 1 (weight 0). */
__global__ __launch_bounds__(PACK_THREADS) void bl_abs_sum_partial_any(const float* __restrict__ W, int64_t count,
                                                                        double* __restrict__ partial) {
    __shared__ double red[PACK_THREADS];
    const int64_t per = (count + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x;
    const int64_t hi = lo + per < count ? lo + per : count;
    double s = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += PACK_THREADS) s += (double)fabsf(W[i]);
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = PACK_THREADS / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

/* One thread = one packed word = 16 consecutive k of one padded row.  IN = 0: fp32 latent
 * weights, ternarised here; IN = 1: int8 ternary weights. */
template <int LAYOUT, int IN>
__global__ __launch_bounds__(PACK_THREADS) void bl_pack_any(const void* __restrict__ Wv, const float* __restrict__ beta,
                                                             int64_t N, int64_t K, int64_t wpr, int64_t words,
                                                             uint32_t* __restrict__ packed) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const int64_t n = g / wpr, k0 = (g % wpr) * 16;
    const float d = IN == 0 ? *beta + 1e-5f : 1.0f;
    int c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t k = k0 + i;
        int t = 0;
        if (n < N && k < K) {
            if (IN == 0) {
                float f = rintf(bl_div_rn(((const float*)Wv)[n * K + k], d));
                f = fminf(fmaxf(f, -1.0f), 1.0f);
                t = (int)f;
            } else {
                const int b = ((const int8_t*)Wv)[n * K + k];
                t = b < -1 ? -1 : (b > 1 ? 1 : b);
            }
        }
        c[i] = t + 1;
    }
    packed[g] = bl_code_word<LAYOUT>(c);
}

template <int LAYOUT>
__global__ __launch_bounds__(PACK_THREADS) void bl_unpack_any(const uint32_t* __restrict__ packed, int64_t N, int64_t K,
                                                               int64_t wpr, int64_t words, int8_t* __restrict__ Wt,
                                                               int32_t* __restrict__ bad) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const int64_t n = g / wpr, k0 = (g % wpr) * 16;
    if (n >= N) return;
    const uint32_t w = packed[g];
    int nbad = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = (int)((w >> bl_bitpos<LAYOUT>(i)) & 3u);
        if (k0 + i < K) {
            nbad += (c == 3);
            Wt[n * K + k0 + i] = (int8_t)(c - 1);
        }
    }
    if (nbad) atomicAdd(bad, nbad);
}

/* ---- five weights per byte (BL_LAYOUT_TRIT5, see bitlinear.h) -----------------------------------
 * One thread = one 4-byte word = 20 consecutive k of one padded row; byte j of the word holds
 * k = 20g + 4i + j, i = 0..4, leading digit first. */
template <int IN>
__global__ __launch_bounds__(PACK_THREADS) void bl_pack_t5(const void* __restrict__ Wv, const float* __restrict__ beta,
                                                            int64_t N, int64_t K, int64_t wpr, int64_t words,
                                                            uint32_t* __restrict__ packed) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const int64_t n = g / wpr, k0 = (g % wpr) * 20;
    const float d = IN == 0 ? *beta + 1e-5f : 1.0f;
    uint32_t word = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t v = 0;
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            const int64_t k = k0 + 4 * i + j;
            int t = 0;
            if (n < N && k < K) {
                if (IN == 0) {
                    float f = rintf(bl_div_rn(((const float*)Wv)[n * K + k], d));
                    f = fminf(fmaxf(f, -1.0f), 1.0f);
                    t = (int)f;
                } else {
                    const int b = ((const int8_t*)Wv)[n * K + k];
                    t = b < -1 ? -1 : (b > 1 ? 1 : b);
                }
            }
            v = v * 3 + (uint32_t)(t + 1);
        }
        word |= ((v * 256 + 242) / 243) << (8 * j);
    }
    packed[g] = word;
}

__global__ __launch_bounds__(PACK_THREADS) void bl_unpack_t5(const uint32_t* __restrict__ packed, int64_t N, int64_t K,
                                                              int64_t wpr, int64_t words, int8_t* __restrict__ Wt,
                                                              int32_t* __restrict__ bad) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const int64_t n = g / wpr, k0 = (g % wpr) * 20;
    if (n >= N) return;
    const uint32_t w = packed[g];
    int nbad = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t b = (w >> (8 * j)) & 0xFFu;
        uint32_t r = b, v = 0;
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            const uint32_t t = r * 3;
            const int c = (int)(t >> 8);
            r = t & 0xFFu;
            v = v * 3 + (uint32_t)c;
            const int64_t k = k0 + 4 * i + j;
            if (k < K) Wt[n * K + k] = (int8_t)(c - 1);
        }
        nbad += ((v * 256 + 242) / 243 != b);          /* a byte that is not the code of its own digits */
    }
    if (nbad) atomicAdd(bad, nbad);
}

/* ---- k-major form (BL_LAYOUT_KMAJOR, see bitlinear.h): the transposed matrix, one row per k ------
 * One thread = one packed word = 16 consecutive n of one k. */
template <int IN>
__global__ __launch_bounds__(PACK_THREADS) void bl_pack_km(const void* __restrict__ Wv, const float* __restrict__ beta,
                                                            int64_t N, int64_t K, int64_t wpr, int64_t words,
                                                            uint32_t* __restrict__ packed) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const int64_t k = g / wpr, n0 = (g % wpr) * 16;
    const float d = IN == 0 ? *beta + 1e-5f : 1.0f;
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t n = n0 + i;
        int t = 0;
        if (n < N) {
            if (IN == 0) {
                float f = rintf(bl_div_rn(((const float*)Wv)[n * K + k], d));
                f = fminf(fmaxf(f, -1.0f), 1.0f);
                t = (int)f;
            } else {
                const int b = ((const int8_t*)Wv)[n * K + k];
                t = b < -1 ? -1 : (b > 1 ? 1 : b);
            }
        }
        word |= (uint32_t)(t + 1) << (2 * i);
    }
    packed[g] = word;
}

__global__ __launch_bounds__(PACK_THREADS) void bl_unpack_km(const uint32_t* __restrict__ packed, int64_t N, int64_t K,
                                                              int64_t wpr, int64_t words, int8_t* __restrict__ Wt,
                                                              int32_t* __restrict__ bad) {
    const int64_t g = (int64_t)blockIdx.x * PACK_THREADS + threadIdx.x;
    if (g >= words) return;
    const int64_t k = g / wpr, n0 = (g % wpr) * 16;
    const uint32_t w = packed[g];
    int nbad = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = (int)((w >> (2 * i)) & 3u);
        if (n0 + i < N) {
            nbad += (c == 3);
            Wt[(n0 + i) * K + k] = (int8_t)(c - 1);
        }
    }
    if (nbad) atomicAdd(bad, nbad);
}

__global__ void bl_zero_i32(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

extern "C" bl_status bl_pack_ternary(const void* W, int in_kind, int64_t N, int64_t K, int layout,
                                     uint8_t* packed, float* beta, void* workspace, bl_stream s) {
    if (!W || !packed || !beta) return BL_ERR_NULL;
    if (!bl_shape_ok(N, K)) return BL_ERR_SHAPE;
    if (layout < BL_LAYOUT_ROWMAJOR || layout > BL_LAYOUT_KMAJOR) return BL_ERR_LAYOUT;
    if (in_kind != BL_IN_FP32_LATENT && in_kind != BL_IN_INT8_TERNARY) return BL_ERR_VALUE;
    if (!bl_aligned(W, 16) || !bl_aligned(packed, 16) || !bl_aligned(beta, 4)) return BL_ERR_ALIGN;
    hipStream_t st = (hipStream_t)s;
    if (layout == BL_LAYOUT_TRIT5 || layout == BL_LAYOUT_KMAJOR) {
        const bool km = layout == BL_LAYOUT_KMAJOR;
        const int64_t wpr = km ? (N + 63) / 64 * 4 : bl_kpad5(K) / 20, pwords = (km ? K : bl_npad(N)) * wpr;
        const unsigned pgrid = (unsigned)((pwords + PACK_THREADS - 1) / PACK_THREADS);
        uint32_t* out = (uint32_t*)packed;
        if (in_kind == BL_IN_FP32_LATENT) {
            if (!workspace) return BL_ERR_WORKSPACE;
            if (!bl_aligned(workspace, 8)) return BL_ERR_ALIGN;
            double* partial = (double*)workspace;
            const int64_t count = N * K;
            const int np = (int)(count < BL_PACK_PARTIALS ? count : BL_PACK_PARTIALS);
            bl_abs_sum_partial_any<<<np, PACK_THREADS, 0, st>>>((const float*)W, count, partial);
            bl_abs_sum_final<<<1, PACK_THREADS, 0, st>>>(partial, np, (double)count, beta);
            if (km) bl_pack_km<0><<<pgrid, PACK_THREADS, 0, st>>>(W, beta, N, K, wpr, pwords, out);
            else bl_pack_t5<0><<<pgrid, PACK_THREADS, 0, st>>>(W, beta, N, K, wpr, pwords, out);
        } else {
            if (km) bl_pack_km<1><<<pgrid, PACK_THREADS, 0, st>>>(W, beta, N, K, wpr, pwords, out);
            else bl_pack_t5<1><<<pgrid, PACK_THREADS, 0, st>>>(W, beta, N, K, wpr, pwords, out);
        }
        return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
    }
    if (!bl_shape_unpadded(N, K)) {
        const int64_t wpr = bl_kpad(K) / 16, pwords = bl_npad(N) * wpr;
        const unsigned pgrid = (unsigned)((pwords + PACK_THREADS - 1) / PACK_THREADS);
        uint32_t* out = (uint32_t*)packed;
        if (in_kind == BL_IN_FP32_LATENT) {
            if (!workspace) return BL_ERR_WORKSPACE;
            if (!bl_aligned(workspace, 8)) return BL_ERR_ALIGN;
            double* partial = (double*)workspace;
            const int64_t count = N * K;
            const int np = (int)(count < BL_PACK_PARTIALS ? count : BL_PACK_PARTIALS);
            bl_abs_sum_partial_any<<<np, PACK_THREADS, 0, st>>>((const float*)W, count, partial);
            bl_abs_sum_final<<<1, PACK_THREADS, 0, st>>>(partial, np, (double)count, beta);
            if (layout == 0) bl_pack_any<0, 0><<<pgrid, PACK_THREADS, 0, st>>>(W, beta, N, K, wpr, pwords, out);
            else bl_pack_any<1, 0><<<pgrid, PACK_THREADS, 0, st>>>(W, beta, N, K, wpr, pwords, out);
        } else {
            if (layout == 0) bl_pack_any<0, 1><<<pgrid, PACK_THREADS, 0, st>>>(W, beta, N, K, wpr, pwords, out);
            else bl_pack_any<1, 1><<<pgrid, PACK_THREADS, 0, st>>>(W, beta, N, K, wpr, pwords, out);
        }
        return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
    }
    const int64_t words = N * K / 16;
    const unsigned grid = (unsigned)((words + PACK_THREADS - 1) / PACK_THREADS);
    if (in_kind == BL_IN_FP32_LATENT) {
        if (!workspace) return BL_ERR_WORKSPACE;
        if (!bl_aligned(workspace, 8)) return BL_ERR_ALIGN;
        double* partial = (double*)workspace;
        const int64_t n4 = N * K / 4;
        const int np = (int)(n4 < BL_PACK_PARTIALS ? n4 : BL_PACK_PARTIALS);
        bl_abs_sum_partial<<<np, PACK_THREADS, 0, st>>>((const float4*)W, n4, partial);
        bl_abs_sum_final<<<1, PACK_THREADS, 0, st>>>(partial, np, (double)(N * K), beta);
        if (layout == 0)
            bl_ternarize_pack<0><<<grid, PACK_THREADS, 0, st>>>((const float4*)W, beta, words, (uint32_t*)packed);
        else
            bl_ternarize_pack<1><<<grid, PACK_THREADS, 0, st>>>((const float4*)W, beta, words, (uint32_t*)packed);
    } else {
        if (layout == 0)
            bl_pack_int8<0><<<grid, PACK_THREADS, 0, st>>>((const bl_v4i*)W, words, (uint32_t*)packed);
        else
            bl_pack_int8<1><<<grid, PACK_THREADS, 0, st>>>((const bl_v4i*)W, words, (uint32_t*)packed);
    }
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

extern "C" bl_status bl_unpack_ternary(const uint8_t* packed, int64_t N, int64_t K, int layout,
                                       int8_t* Wt, int32_t* bad, bl_stream s) {
    if (!packed || !Wt || !bad) return BL_ERR_NULL;
    if (!bl_shape_ok(N, K)) return BL_ERR_SHAPE;
    if (layout < BL_LAYOUT_ROWMAJOR || layout > BL_LAYOUT_KMAJOR) return BL_ERR_LAYOUT;
    if (!bl_aligned(packed, 16) || !bl_aligned(Wt, 16) || !bl_aligned(bad, 4)) return BL_ERR_ALIGN;
    hipStream_t st = (hipStream_t)s;
    if (layout == BL_LAYOUT_TRIT5 || layout == BL_LAYOUT_KMAJOR) {
        const bool km = layout == BL_LAYOUT_KMAJOR;
        const int64_t wpr = km ? (N + 63) / 64 * 4 : bl_kpad5(K) / 20, pwords = (km ? K : bl_npad(N)) * wpr;
        const unsigned pgrid = (unsigned)((pwords + PACK_THREADS - 1) / PACK_THREADS);
        bl_zero_i32<<<1, 64, 0, st>>>(bad, 1);
        if (km) bl_unpack_km<<<pgrid, PACK_THREADS, 0, st>>>((const uint32_t*)packed, N, K, wpr, pwords, Wt, bad);
        else bl_unpack_t5<<<pgrid, PACK_THREADS, 0, st>>>((const uint32_t*)packed, N, K, wpr, pwords, Wt, bad);
        return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
    }
    if (!bl_shape_unpadded(N, K)) {
        const int64_t wpr = bl_kpad(K) / 16, pwords = bl_npad(N) * wpr;
        const unsigned pgrid = (unsigned)((pwords + PACK_THREADS - 1) / PACK_THREADS);
        bl_zero_i32<<<1, 64, 0, st>>>(bad, 1);
        if (layout == 0) bl_unpack_any<0><<<pgrid, PACK_THREADS, 0, st>>>((const uint32_t*)packed, N, K, wpr, pwords, Wt, bad);
        else bl_unpack_any<1><<<pgrid, PACK_THREADS, 0, st>>>((const uint32_t*)packed, N, K, wpr, pwords, Wt, bad);
        return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
    }
    const int64_t words = N * K / 16;
    const unsigned grid = (unsigned)((words + PACK_THREADS - 1) / PACK_THREADS);
    bl_zero_i32<<<1, 64, 0, st>>>(bad, 1);
    if (layout == 0)
        bl_unpack_kernel<0><<<grid, PACK_THREADS, 0, st>>>((const uint32_t*)packed, words, (bl_v4i*)Wt, bad);
    else
        bl_unpack_kernel<1><<<grid, PACK_THREADS, 0, st>>>((const uint32_t*)packed, words, (bl_v4i*)Wt, bad);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}
