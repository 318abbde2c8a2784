/* Fused producers: the elementwise step that yields the bf16 input of a
 * BitLinear, evaluated inside the kernel that quantises it, so the bf16 tensor
 * never exists in HBM.  Each kind is exact elementwise fp32 work followed by a
 * round-to-nearest-even narrowing to bf16 (ReLU^2 in the FFN is the report's,
 * Section 2; the residual add and the context-length-1 attention are the
 * synthetic chain glue of this repository). */
#pragma once
#include "bl_device.h"

struct bl_prod_dev {
    int kind;            /* BL_PROD_* */
    const void* in0;
    const float* in1;
    float* aux_out;
    int voff, group, hd, in_stride;   /* ATTN_V geometry; in_stride = floats per source row */
    int norm;            /* RMS normalisation in front of the quantiser */
    const float* gain;   /* [K] or NULL */
    float eps;
};

__device__ __forceinline__ uint32_t bl_pack2_bf16(float a, float b) {
    return bl_f32_to_bf16(a) | (bl_f32_to_bf16(b) << 16);
}

/* fp32 values of k = 16u .. 16u+15 of token m, before narrowing (any kind).
 * store_aux: this caller also writes the fp32 by-product (RESIDUAL: the sum). */
__device__ __forceinline__ void bl_produce16_f32(const bl_prod_dev& pd, int m, int u, int K, bool store_aux,
                                                 float v[16]) {
    if (pd.kind == BL_PROD_BF16) {
        const uint4* xr = (const uint4*)((const uint16_t*)pd.in0 + (int64_t)m * K);
        const uint4 lo = xr[2 * u], hi = xr[2 * u + 1];
        const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            v[2 * j] = bl_bf16_to_f32(w[j] & 0xFFFFu);
            v[2 * j + 1] = bl_bf16_to_f32(w[j] >> 16);
        }
        return;
    }
    if (pd.kind == BL_PROD_RELU2_GATE) {
        const float4* g4 = (const float4*)((const float*)pd.in0 + (int64_t)m * 2 * K + (int64_t)u * 16);
        const float4* u4 = (const float4*)((const float*)pd.in0 + (int64_t)m * 2 * K + K + (int64_t)u * 16);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 g = g4[j], up = u4[j];
            const float gg[4] = {g.x, g.y, g.z, g.w}, uu[4] = {up.x, up.y, up.z, up.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float r = fmaxf(gg[e], 0.0f);
                const float r2 = r * r;
                v[4 * j + e] = r2 * uu[e];
            }
        }
        return;
    }
    int64_t off;
    if (pd.kind == BL_PROD_ATTN_V) {
        const int k = u * 16;
        off = (int64_t)m * pd.in_stride + pd.voff + ((k / pd.hd) / pd.group) * pd.hd + (k % pd.hd);
    } else {
        off = (int64_t)m * K + (int64_t)u * 16;
    }
    const float4* a4 = (const float4*)((const float*)pd.in0 + off);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float4 a = a4[j];
        v[4 * j] = a.x; v[4 * j + 1] = a.y; v[4 * j + 2] = a.z; v[4 * j + 3] = a.w;
    }
    if (pd.kind == BL_PROD_RESIDUAL) {
        const float4* b4 = (const float4*)(pd.in1 + off);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 b = b4[j];
            v[4 * j] += b.x; v[4 * j + 1] += b.y; v[4 * j + 2] += b.z; v[4 * j + 3] += b.w;
        }
        if (store_aux && pd.aux_out) {
            float4* o4 = (float4*)(pd.aux_out + off);
#pragma unroll
            for (int j = 0; j < 4; ++j) o4[j] = make_float4(v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]);
        }
    }
}

/* bf16 bit patterns of k = 16u .. 16u+15 of token m: lo = first eight, hi = last eight.
 * rn: the token's normalisation factor (used only if NORM and pd.norm).  NORM = false
 * compiles the normalisation out: kernels that never normalise keep their registers. */
template <bool NORM>
__device__ __forceinline__ void bl_produce16(const bl_prod_dev& pd, int m, int u, int K, bool store_aux, float rn,
                                             uint4& lo, uint4& hi) {
    if (pd.kind == BL_PROD_BF16 && !(NORM && pd.norm)) {
        const uint4* xr = (const uint4*)((const uint16_t*)pd.in0 + (int64_t)m * K);
        lo = xr[2 * u];
        hi = xr[2 * u + 1];
        return;
    }
    float v[16];
    bl_produce16_f32(pd, m, u, K, store_aux, v);
    if (NORM && pd.norm) {
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = v[e] * rn;
        if (pd.gain) {
            const float4* g4 = (const float4*)(pd.gain + (int64_t)u * 16);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float4 g = g4[j];
                v[4 * j] *= g.x; v[4 * j + 1] *= g.y; v[4 * j + 2] *= g.z; v[4 * j + 3] *= g.w;
            }
        }
    }
    lo = make_uint4(bl_pack2_bf16(v[0], v[1]), bl_pack2_bf16(v[2], v[3]), bl_pack2_bf16(v[4], v[5]),
                    bl_pack2_bf16(v[6], v[7]));
    hi = make_uint4(bl_pack2_bf16(v[8], v[9]), bl_pack2_bf16(v[10], v[11]), bl_pack2_bf16(v[12], v[13]),
                    bl_pack2_bf16(v[14], v[15]));
}

/* Normalising production of token m by a 256-thread workgroup, in the fixed order of the
 * public header (thread j is leaf j).  The thread's first two groups (u = tid, tid + 256) are
 * produced once, kept in registers across the reduction and returned as normalised bf16 words
 * in xv[0..3]; groups beyond those (K > 8192) only enter the sum and are produced again by the
 * caller with the returned factor.  store_aux as in bl_produce16_f32.  s4: four doubles of LDS,
 * free to reuse after the caller's next barrier.  Contains one barrier. */
__device__ __forceinline__ float bl_norm_produce2(const bl_prod_dev& pd, int m, int K, bool store_aux, double* s4,
                                                  uint4 xv[4]) {
    const int tid = threadIdx.x, groups = K / 16;
    float tv[2][16];
    double part = 0.0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int u = tid + j * 256;
        if (u < groups) {
            bl_produce16_f32(pd, m, u, K, store_aux, tv[j]);
#pragma unroll
            for (int e = 0; e < 16; ++e) part += (double)tv[j][e] * (double)tv[j][e];
        }
    }
    for (int u = tid + 512; u < groups; u += 256) {
        float v[16];
        bl_produce16_f32(pd, m, u, K, false, v);
#pragma unroll
        for (int e = 0; e < 16; ++e) part += (double)v[e] * (double)v[e];
    }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) part += __shfl_xor(part, s);
    if ((tid & 63) == 0) s4[tid >> 6] = part;
    __syncthreads();
    const double ss = (s4[0] + s4[1]) + (s4[2] + s4[3]);
    const float rn = (float)(1.0 / sqrt(ss / (double)K + (double)pd.eps));
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int u = tid + j * 256;
        if (u < groups) {
            float* v = tv[j];
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] = v[e] * rn;
            if (pd.gain) {
                const float4* g4 = (const float4*)(pd.gain + (int64_t)u * 16);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 g = g4[q];
                    v[4 * q] *= g.x; v[4 * q + 1] *= g.y; v[4 * q + 2] *= g.z; v[4 * q + 3] *= g.w;
                }
            }
            xv[2 * j] = make_uint4(bl_pack2_bf16(v[0], v[1]), bl_pack2_bf16(v[2], v[3]), bl_pack2_bf16(v[4], v[5]),
                                   bl_pack2_bf16(v[6], v[7]));
            xv[2 * j + 1] = make_uint4(bl_pack2_bf16(v[8], v[9]), bl_pack2_bf16(v[10], v[11]),
                                       bl_pack2_bf16(v[12], v[13]), bl_pack2_bf16(v[14], v[15]));
        }
    }
    return rn;
}

/* Quantise 8 bf16 (one uint4) to two dwords of int8: q = clamp(rint(x*inv), -127, 127). */
__device__ __forceinline__ void bl_quant8_words(const uint4 v, float inv, uint32_t& lo, uint32_t& hi) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[2] = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t hbits = (j & 1) ? (w[j >> 1] >> 16) : (w[j >> 1] & 0xFFFFu);
        float r = rintf(bl_bf16_to_f32(hbits) * inv);
        r = fminf(fmaxf(r, -127.0f), 127.0f);
        o[j >> 2] |= ((uint32_t)(int)r & 0xFFu) << (8 * (j & 3));
    }
    lo = o[0];
    hi = o[1];
}

__device__ __forceinline__ float bl_absmax8_bf16(const uint4 v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        m = fmaxf(m, fabsf(bl_bf16_to_f32(w[j] & 0xFFFFu)));
        m = fmaxf(m, fabsf(bl_bf16_to_f32(w[j] >> 16)));
    }
    return m;
}

__device__ __forceinline__ int bl_sum16(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3) {
    int part = __builtin_amdgcn_sdot4((int)a0, 0x01010101, 0, false);
    part = __builtin_amdgcn_sdot4((int)a1, 0x01010101, part, false);
    part = __builtin_amdgcn_sdot4((int)a2, 0x01010101, part, false);
    return __builtin_amdgcn_sdot4((int)a3, 0x01010101, part, false);
}

/* Host side: public descriptor -> device form.  Returns false on a bad descriptor. */
static inline bool bl_make_prod(const bl_producer& p, const uint16_t* x_default, int64_t K, bl_prod_dev* out) {
    bl_prod_dev d = {};
    d.kind = p.kind;
    d.in0 = p.in0 ? p.in0 : (const void*)x_default;
    d.in1 = p.in1;
    d.aux_out = p.aux_out;
    d.norm = p.norm ? 1 : 0;
    d.gain = p.norm ? p.gain : nullptr;
    d.eps = p.eps;
    if (!d.in0) return false;
    if (p.norm && !(p.eps >= 0.0f)) return false;
    if (p.kind < BL_PROD_BF16 || p.kind > BL_PROD_RELU2_GATE) return false;
    if (p.kind == BL_PROD_RESIDUAL && !p.in1) return false;
    if (p.kind == BL_PROD_ATTN_V) {
        if (p.n_q <= 0 || p.n_kv <= 0 || p.head_dim <= 0 || p.n_q % p.n_kv || p.head_dim % 16 ||
            (int64_t)p.n_q * p.head_dim != K)
            return false;
        d.voff = (p.n_q + p.n_kv) * p.head_dim;
        d.group = p.n_q / p.n_kv;
        d.hd = p.head_dim;
        d.in_stride = (p.n_q + 2 * p.n_kv) * p.head_dim;
    }
    if (((uintptr_t)d.in0 | (uintptr_t)d.in1 | (uintptr_t)d.aux_out | (uintptr_t)d.gain) & 15) return false;
    *out = d;
    return true;
}
