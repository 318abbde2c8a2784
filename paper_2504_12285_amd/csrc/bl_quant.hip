/* Per-token absmax int8 activation quantisation (Section 2, "Activation
 * Quantization", of the BitNet b1.58 2B4T report).  One workgroup per token
 * row; the row is read twice (absmax, then quantise), the second pass hitting
 * cache.  HBM-bound at prefill sizes, latency-bound at decode sizes. */
#include "bl_device.h"
#include "bl_host.h"
#include "bl_producer.h"

#define QUANT_THREADS 256

/* Quantise 8 bf16 values held in a uint4 to 8 int8 in a uint2; returns their sum. */
__device__ __forceinline__ int bl_quant8(const uint4 v, float inv, uint2* out) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[2] = {0u, 0u};
    int sum = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t h = (j & 1) ? (w[j >> 1] >> 16) : (w[j >> 1] & 0xFFFFu);
        float r = rintf(bl_bf16_to_f32(h) * inv);
        r = fminf(fmaxf(r, -127.0f), 127.0f);
        const int qi = (int)r;
        sum += qi;
        o[j >> 2] |= ((uint32_t)qi & 0xFFu) << (8 * (j & 3));
    }
    out->x = o[0];
    out->y = o[1];
    return sum;
}

__device__ __forceinline__ float bl_absmax8(const uint4 v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        m = fmaxf(m, fabsf(bl_bf16_to_f32(w[j] & 0xFFFFu)));
        m = fmaxf(m, fabsf(bl_bf16_to_f32(w[j] >> 16)));
    }
    return m;
}

__global__ __launch_bounds__(QUANT_THREADS) void bl_quant_rows(const uint4* __restrict__ X, int K8,
                                                                uint2* __restrict__ q, float* __restrict__ scale,
                                                                int32_t* __restrict__ rowsum) {
    __shared__ float smax[QUANT_THREADS / BL_WAVE];
    __shared__ int ssum[QUANT_THREADS / BL_WAVE];
    const int64_t m = blockIdx.x;
    const uint4* x = X + m * K8;
    uint2* qo = q + m * K8;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;

    float mx = 0.0f;
    for (int i = threadIdx.x; i < K8; i += QUANT_THREADS) mx = fmaxf(mx, bl_absmax8(x[i]));
    mx = bl_wave_max(mx);
    if (lane == 0) smax[w] = mx;
    __syncthreads();
    float gamma = smax[0];
#pragma unroll
    for (int i = 1; i < QUANT_THREADS / BL_WAVE; ++i) gamma = fmaxf(gamma, smax[i]);

    const float g = fmaxf(gamma, 1e-5f);
    const float inv = bl_div_rn(127.0f, g);
    int sum = 0;
    for (int i = threadIdx.x; i < K8; i += QUANT_THREADS) {
        uint2 o;
        sum += bl_quant8(x[i], inv, &o);
        qo[i] = o;
    }
    sum = bl_wave_sum(sum);
    if (lane == 0) ssum[w] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        scale[m] = bl_div_rn(g, 127.0f);
        if (rowsum) {
            int t = 0;
#pragma unroll
            for (int i = 0; i < QUANT_THREADS / BL_WAVE; ++i) t += ssum[i];
            rowsum[m] = t;
        }
    }
}

/* The same quantiser for a ragged K (not a multiple of 64): element-wise reads of the bf16 row
 * (its start need not be 16-byte aligned), output row of Kp = ceil(K/64)*64 bytes with zeros in
 * the padding. */
__global__ __launch_bounds__(QUANT_THREADS) void bl_quant_rows_any(const uint16_t* __restrict__ X, int K, int Kp,
                                                                    int8_t* __restrict__ q, float* __restrict__ scale,
                                                                    int32_t* __restrict__ rowsum) {
    __shared__ float smax[QUANT_THREADS / BL_WAVE];
    __shared__ int ssum[QUANT_THREADS / BL_WAVE];
    const int64_t m = blockIdx.x;
    const uint16_t* x = X + m * K;
    int8_t* qo = q + m * Kp;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    float mx = 0.0f;
    for (int i = threadIdx.x; i < K; i += QUANT_THREADS) mx = fmaxf(mx, fabsf(bl_bf16_to_f32(x[i])));
    mx = bl_wave_max(mx);
    if (lane == 0) smax[w] = mx;
    __syncthreads();
    float gamma = smax[0];
#pragma unroll
    for (int i = 1; i < QUANT_THREADS / BL_WAVE; ++i) gamma = fmaxf(gamma, smax[i]);
    const float g = fmaxf(gamma, 1e-5f);
    const float inv = bl_div_rn(127.0f, g);
    int sum = 0;
    for (int i = threadIdx.x; i < Kp; i += QUANT_THREADS) {
        int qi = 0;
        if (i < K) {
            float r = rintf(bl_bf16_to_f32(x[i]) * inv);
            r = fminf(fmaxf(r, -127.0f), 127.0f);
            qi = (int)r;
        }
        sum += qi;
        qo[i] = (int8_t)qi;
    }
    sum = bl_wave_sum(sum);
    if (lane == 0) ssum[w] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        scale[m] = bl_div_rn(g, 127.0f);
        if (rowsum) {
            int t = 0;
#pragma unroll
            for (int i = 0; i < QUANT_THREADS / BL_WAVE; ++i) t += ssum[i];
            rowsum[m] = t;
        }
    }
}

/* Producer + quantiser: the bf16 row is produced on the fly (bl_produce16) and
 * kept in registers between the absmax pass and the quantise pass (two
 * 16-element groups per thread cover K <= 8192; longer rows are produced twice). */
template <bool NORM>
__global__ __launch_bounds__(QUANT_THREADS) void bl_quant_rows_ex(const bl_prod_dev pd, int K,
                                                                   int8_t* __restrict__ q, float* __restrict__ scale,
                                                                   int32_t* __restrict__ rowsum) {
    __shared__ float smax[QUANT_THREADS / BL_WAVE];
    __shared__ int ssum[QUANT_THREADS / BL_WAVE];
    __shared__ double snorm[4];
    static_assert(QUANT_THREADS == 256, "the normalisation tree has 256 leaves");
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int groups = K / 16;
    uint4 xv[4];
    float rn = 1.0f;
    if (NORM) rn = bl_norm_produce2(pd, m, K, true, snorm, xv);
    float mx = 0.0f;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int u = tid + j * QUANT_THREADS;
        if (u < groups) {
            if (!NORM) bl_produce16<NORM>(pd, m, u, K, true, rn, xv[2 * j], xv[2 * j + 1]);
            mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(xv[2 * j]), bl_absmax8_bf16(xv[2 * j + 1])));
        }
    }
    for (int u = tid + 2 * QUANT_THREADS; u < groups; u += QUANT_THREADS) {
        uint4 lo, hi;
        bl_produce16<NORM>(pd, m, u, K, true, rn, lo, hi);
        mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(lo), bl_absmax8_bf16(hi)));
    }
    mx = bl_wave_max(mx);
    if (lane == 0) smax[w] = mx;
    __syncthreads();
    float gamma = smax[0];
#pragma unroll
    for (int i = 1; i < QUANT_THREADS / BL_WAVE; ++i) gamma = fmaxf(gamma, smax[i]);
    const float g = fmaxf(gamma, 1e-5f);
    const float inv = bl_div_rn(127.0f, g);
    int8_t* qo = q + (int64_t)m * K;
    int sum = 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int u = tid + j * QUANT_THREADS;
        if (u < groups) {
            uint32_t a0, a1, a2, a3;
            bl_quant8_words(xv[2 * j], inv, a0, a1);
            bl_quant8_words(xv[2 * j + 1], inv, a2, a3);
            sum += bl_sum16(a0, a1, a2, a3);
            *(uint4*)(qo + u * 16) = make_uint4(a0, a1, a2, a3);
        }
    }
    for (int u = tid + 2 * QUANT_THREADS; u < groups; u += QUANT_THREADS) {
        uint4 lo, hi;
        uint32_t a0, a1, a2, a3;
        bl_produce16<NORM>(pd, m, u, K, false, rn, lo, hi);
        bl_quant8_words(lo, inv, a0, a1);
        bl_quant8_words(hi, inv, a2, a3);
        sum += bl_sum16(a0, a1, a2, a3);
        *(uint4*)(qo + u * 16) = make_uint4(a0, a1, a2, a3);
    }
    sum = bl_wave_sum(sum);
    if (lane == 0) ssum[w] = sum;
    __syncthreads();
    if (tid == 0) {
        scale[m] = bl_div_rn(g, 127.0f);
        if (rowsum) {
            int t = 0;
#pragma unroll
            for (int i = 0; i < QUANT_THREADS / BL_WAVE; ++i) t += ssum[i];
            rowsum[m] = t;
        }
    }
}

extern "C" bl_status bl_quant_act_ex(const bl_producer* prod, int64_t M, int64_t K, int8_t* q, float* scale,
                                     int32_t* rowsum, bl_stream s) {
    if (!prod || !q || !scale) return BL_ERR_NULL;
    if (M < 1 || M > BL_MAX_DIM || K < 64 || K % 64 != 0 || K > BL_MAX_DIM) return BL_ERR_SHAPE;
    if (!bl_aligned(q, 16) || !bl_aligned(scale, 4) || !bl_aligned(rowsum, 4)) return BL_ERR_ALIGN;
    bl_prod_dev pd;
    if (!prod->in0) return BL_ERR_NULL;
    if (!bl_make_prod(*prod, nullptr, K, &pd)) return BL_ERR_VALUE;
    if (pd.norm) bl_quant_rows_ex<true><<<(unsigned)M, QUANT_THREADS, 0, (hipStream_t)s>>>(pd, (int)K, q, scale, rowsum);
    else bl_quant_rows_ex<false><<<(unsigned)M, QUANT_THREADS, 0, (hipStream_t)s>>>(pd, (int)K, q, scale, rowsum);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

/* Quantiser behind a fused producer epilogue: the bf16 row and its absmax already exist, so one
 * pass quantises.  absmax[m] holds the float bits of max_k |x|; it is read by every thread and then
 * cleared, so that the next product's epilogue can fold its maxima into it again. */
__global__ __launch_bounds__(QUANT_THREADS) void bl_quant_rows_absmax(const uint4* __restrict__ X, int K8,
                                                                       int* __restrict__ absmax,
                                                                       uint2* __restrict__ q, float* __restrict__ scale,
                                                                       int32_t* __restrict__ rowsum) {
    __shared__ int ssum[QUANT_THREADS / BL_WAVE];
    const int64_t m = blockIdx.x;
    const uint4* x = X + m * K8;
    uint2* qo = q + m * K8;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const float gamma = __int_as_float(absmax[m]);
    const float g = fmaxf(gamma, 1e-5f);
    const float inv = bl_div_rn(127.0f, g);
    int sum = 0;
    for (int i = threadIdx.x; i < K8; i += QUANT_THREADS) {
        uint2 o;
        sum += bl_quant8(x[i], inv, &o);
        qo[i] = o;
    }
    sum = bl_wave_sum(sum);
    if (lane == 0) ssum[w] = sum;
    __syncthreads();                      /* every thread has read absmax[m] */
    if (threadIdx.x == 0) {
        absmax[m] = 0;
        scale[m] = bl_div_rn(g, 127.0f);
        if (rowsum) {
            int t = 0;
#pragma unroll
            for (int i = 0; i < QUANT_THREADS / BL_WAVE; ++i) t += ssum[i];
            rowsum[m] = t;
        }
    }
}

extern "C" bl_status bl_quant_from_absmax(const uint16_t* X, float* absmax, int64_t M, int64_t K, int8_t* q,
                                          float* scale, int32_t* rowsum, bl_stream s) {
    if (!X || !absmax || !q || !scale) return BL_ERR_NULL;
    if (M < 1 || M > BL_MAX_DIM || K < 64 || K % 64 != 0 || K > BL_MAX_DIM) return BL_ERR_SHAPE;
    if (!bl_aligned(X, 16) || !bl_aligned(q, 16) || !bl_aligned(scale, 4) || !bl_aligned(rowsum, 4) ||
        !bl_aligned(absmax, 4))
        return BL_ERR_ALIGN;
    bl_quant_rows_absmax<<<(unsigned)M, QUANT_THREADS, 0, (hipStream_t)s>>>((const uint4*)X, (int)(K / 8), (int*)absmax,
                                                                           (uint2*)q, scale, rowsum);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

extern "C" bl_status bl_quant_act_int8(const uint16_t* X, int64_t M, int64_t K, int8_t* q, float* scale,
                                       int32_t* rowsum, bl_stream s) {
    if (!X || !q || !scale) return BL_ERR_NULL;
    if (M < 1 || M > BL_MAX_DIM || K < 1 || K > BL_MAX_DIM) return BL_ERR_SHAPE;
    if (K % 64 != 0) {
        if (!bl_aligned(X, 2) || !bl_aligned(q, 16) || !bl_aligned(scale, 4) || !bl_aligned(rowsum, 4))
            return BL_ERR_ALIGN;
        bl_quant_rows_any<<<(unsigned)M, QUANT_THREADS, 0, (hipStream_t)s>>>(X, (int)K, (int)bl_kpad(K), q, scale, rowsum);
        return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
    }
    if (!bl_aligned(X, 16) || !bl_aligned(q, 16) || !bl_aligned(scale, 4) || !bl_aligned(rowsum, 4))
        return BL_ERR_ALIGN;
    bl_quant_rows<<<(unsigned)M, QUANT_THREADS, 0, (hipStream_t)s>>>((const uint4*)X, (int)(K / 8), (uint2*)q,
                                                                    scale, rowsum);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}
