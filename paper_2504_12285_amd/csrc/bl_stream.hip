/* Persistent streaming decode (Section 5.1 of the BitNet b1.58 2B4T report: the decode
 * kernel exists to minimise memory-bandwidth use, so the packed weights of a whole stack of
 * BitLinear products are streamed from HBM in ONE launch whose loads never stop).
 *
 * A table of products lives in device memory.  The grid is as many workgroups as stay
 * resident; each owns one contiguous slice of the table's weight bytes, cut at row-group
 * boundaries, so a workgroup meets one or two products and quantises / stages the activation
 * row of a product once, into LDS.  Inside a product the four waves of a workgroup take row
 * groups round-robin and double-buffer the 128-bit weight loads: the loads of row group i+1
 * are issued before the dot products of row group i.
 *
 * Arithmetic as in bl_gemv.hip: offset codes c = Wt + 1, bit-pair levels isolated by masks,
 * v_dot4_i32_i8 into four accumulators carrying 1, 4, 16, 16, DPP sums over the G lanes of
 * a row, rowsum subtracted once per output.  One token per product (M = 1).
 */
#include <string.h>

#include <atomic>
#include <type_traits>

#include <algorithm>
#include <queue>
#include <vector>

#include "bl_device.h"
#include "bl_gemv_common.h"
#include "bl_host.h"
#include "bl_producer.h"

/* ---- device side -------------------------------------------------------------------------- */

/* Pointers read from the product table are generic to the compiler; they are cast to the
 * global address space so that their loads and stores are global_* instructions with exact
 * counter waits (a generic access forces a full wait at every use). */
#define BL_G __attribute__((address_space(1)))
typedef bl_v4i BL_G bl_gv4i;

/* What the streaming kernel needs to know about one product (device memory). */
struct bl_stream_item {
    const bl_v4i* packed;
    const int8_t* q;          /* [K] int8: the caller's, or the preparation kernel's output */
    const float* scale;       /* [1] token part of the rescale factor (NULL: y is not wanted) */
    const int32_t* rowsum;    /* [1] sum_k q */
    const float* beta;
    const float* residual;    /* [N] or NULL */
    int32_t* acc;             /* [N] or NULL */
    float* y;                 /* [N] or NULL */
    const uint16_t* xbf16;    /* [K] bf16, or NULL: quantised by every workgroup that meets the product */
    int8_t* q_out;            /* xbf16 only: the caller's optional copies of q and absmax/127 */
    float* scale_out;
    float fixed_scale;        /* xbf16 only: > 0 replaces absmax/127 in the rescale */
    int N, nchunks, lgG, lp, layout, units;
    int qgroups;              /* 16-byte groups of the quantised row (its padded length / 16) */
    int m;                    /* tokens of the entry (batched form; 1 otherwise) */
    int row_chunks, c0;       /* batched form: 16-byte chunks of a whole packed row; first chunk of the entry's k part */
    int ldq;                  /* batched form: bytes of a token row of q */
    /* k-major form only: partial sums of all workgroups, and what the finishing kernel reads */
    int32_t* acc_ws;          /* [N] int32, zero between runs */
    const int32_t* rowsum_fin;
    const float* scale_fin;
    int32_t* rowsum_pub;      /* bf16 input: where the owner workgroup publishes sum_k q and the scale */
    float* scale_pub;
};

/* What the preparation kernel needs: the fused producer + quantiser of one product. */
struct bl_stream_prep_item {
    bl_prod_dev prod;
    int fused;                /* 1: produce + quantise; 0: only the row sum of a given q is missing */
    const int8_t* q_in;       /* fused == 0 */
    int8_t* q_ws;             /* [K] quantised row (fused) */
    float* scale_ws;          /* [1] rescale factor's token part (fused) */
    int32_t* rowsum_ws;       /* [1] */
    int8_t* q_out;            /* caller's optional copies */
    float* scale_out;
    float fixed_scale;
    int K;
};

/* Sum over aligned groups of 1 << lgG lanes (8, 16, 32 or 64), result in every lane. */
__device__ __forceinline__ int bl_group_sum_rt(int v, int lgG) {
    v = bl_group_sum<8>(v);
    if (lgG >= 4) v += bl_dpp<BL_DPP_ROW_MIRROR>(v);
    if (lgG >= 5) v += __shfl_xor(v, 16);
    if (lgG >= 6) v += __shfl_xor(v, 32);
    return v;
}

/* The four bit-pair levels of four packed words against the sixteen activation dwords
 * a[s][d] of one chunk. */
__device__ __forceinline__ void bl_stream_dot(const bl_v4i p, const bl_v4i* a, int* A) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t w = (uint32_t)p[d];
            const uint32_t lv = s == 0 ? (w & 0x03030303u)
                              : s == 1 ? (w & 0x0C0C0C0Cu)
                              : s == 2 ? (w & 0x30303030u)
                                       : ((w >> 2) & 0x30303030u);
            A[s] = __builtin_amdgcn_sdot4((int)lv, a[s][d], A[s], false);
        }
    }
}

/* Preparation: one workgroup per table entry that needs it.  Fused entries: producer, RMS
 * normalisation (NORM), per-token absmax, int8 quantisation (Section 2) into the workspace,
 * with the caller's optional copies; int8 entries without a row sum: the row sum. */
template <bool NORM>
__global__ __launch_bounds__(256) void bl_stream_prep(const bl_stream_prep_item* __restrict__ items) {
    __shared__ float fs[4];
    __shared__ int ssum[4];
    __shared__ double s4[4];
    const bl_stream_prep_item& it = items[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int K = it.K, groups = K / 16;
    int part = 0;
    if (it.fused) {
        const bl_prod_dev pd = it.prod;
        uint4 xv[4];
        float rn = 1.0f;
        bool have_xv = false;
        if (NORM && pd.norm) {
            rn = bl_norm_produce2(pd, 0, K, true, s4, xv);
            have_xv = true;
        }
        float mx = 0.0f;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int u = tid + j * 256;
            if (u < groups) {
                if (!have_xv) bl_produce16<NORM>(pd, 0, u, K, true, rn, xv[2 * j], xv[2 * j + 1]);
                mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(xv[2 * j]), bl_absmax8_bf16(xv[2 * j + 1])));
            }
        }
        for (int u = tid + 512; u < groups; u += 256) {
            uint4 lo, hi;
            bl_produce16<NORM>(pd, 0, u, K, false, rn, lo, hi);
            mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(lo), bl_absmax8_bf16(hi)));
        }
        mx = bl_wave_max(mx);
        if (lane == 0) fs[w] = mx;
        __syncthreads();
        const float gamma = fmaxf(fmaxf(fs[0], fs[1]), fmaxf(fs[2], fs[3]));
        const float gg = fmaxf(gamma, 1e-5f);
        const float inv = bl_div_rn(127.0f, gg);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int u = tid + j * 256;
            if (u < groups) {
                uint32_t a0, a1, a2, a3;
                bl_quant8_words(xv[2 * j], inv, a0, a1);
                bl_quant8_words(xv[2 * j + 1], inv, a2, a3);
                part += bl_sum16(a0, a1, a2, a3);
                if (it.q_out) *(uint4*)(it.q_out + u * 16) = make_uint4(a0, a1, a2, a3);
                *(uint4*)(it.q_ws + u * 16) = make_uint4(a0, a1, a2, a3);
            }
        }
        for (int u = tid + 512; u < groups; u += 256) {
            uint32_t a0, a1, a2, a3;
            uint4 lo, hi;
            bl_produce16<NORM>(pd, 0, u, K, true, rn, lo, hi);
            bl_quant8_words(lo, inv, a0, a1);
            bl_quant8_words(hi, inv, a2, a3);
            part += bl_sum16(a0, a1, a2, a3);
            if (it.q_out) *(uint4*)(it.q_out + u * 16) = make_uint4(a0, a1, a2, a3);
            *(uint4*)(it.q_ws + u * 16) = make_uint4(a0, a1, a2, a3);
        }
        if (tid == 0) {
            const float sc = bl_div_rn(gg, 127.0f);
            *it.scale_ws = it.fixed_scale > 0.0f ? it.fixed_scale : sc;
            if (it.scale_out) *it.scale_out = sc;
        }
    } else {
        for (int u = tid; u < groups; u += 256) {
            const uint4 v = *(const uint4*)(it.q_in + (int64_t)u * 16);
            part += bl_sum16(v.x, v.y, v.z, v.w);
        }
    }
    part = bl_wave_sum(part);
    if (lane == 0) ssum[w] = part;
    __syncthreads();
    if (tid == 0) *it.rowsum_ws = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
}

/* ---- the stream kernel ----------------------------------------------------------------------
 * A product's quantised activation row lives in LDS for the workgroup (staged once per product
 * and workgroup: quantised from bf16 right there, or copied from the int8 row) and is read with
 * ds_read_b128 right before each group of sixteen dot products.  Holding the row in registers
 * instead (80 per lane) was measured: 2 waves per SIMD, 5.7 - 5.9 TB/s against 5.85 - 6.2 here
 * with 4; the loop issues ~300 vector instructions per 5 KiB of weights, so the vector unit,
 * not the memory, sets the pace (a plain read with the same access pattern gets 7.0 TB/s).
 * Every workgroup that meets a bf16 product quantises the row for itself: nothing crosses
 * workgroups inside the launch.  (A hand-over through ready flags was measured and dropped:
 * fresh data needs either an L2 write-back + invalidate per wave, +40 us per launch, or
 * uncached loads of the row by every wave, +26 us; a separate preparation launch costs 5.5 us.)
 * LDS image: per 64-wide k chunk 20 dwords (16 + 4 of padding so that the eight chunks a wave
 * reads together fall on different banks), dword s*4+d = the bytes that pair with bit-pair
 * level s of packed word d; one all-zero chunk behind the last for lanes whose load is clamped. */
#define BL_QSTRIDE 20

__device__ __forceinline__ void bl_lds_put16(int* __restrict__ Qs, int c16, int layout, uint32_t a0, uint32_t a1,
                                             uint32_t a2, uint32_t a3) {
    if (layout == 0) bl_transpose4x4(a0, a1, a2, a3);
    int* dst = Qs + (c16 >> 2) * BL_QSTRIDE + (c16 & 3);
    dst[0] = (int)a0;
    dst[4] = (int)a1;
    dst[8] = (int)a2;
    dst[12] = (int)a3;
}

/* Stages the activation row of P: Qs = the image above, misc[0] = sum_k q, misc[1] = token part
 * of the rescale factor (float bits).  Ends with a barrier. */
__device__ __forceinline__ void bl_stream_stage(const bl_stream_item& P, int* __restrict__ Qs,
                                                    int* __restrict__ misc, bool owner) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int groups = P.nchunks * 4;
    float* fs = (float*)(misc + 2);
    int* ssum = misc + 6;
    if (tid < BL_QSTRIDE) Qs[P.nchunks * BL_QSTRIDE + tid] = 0;
    int part = 0;
    if (P.xbf16) {
        const bl_gv4i* x = (const bl_gv4i*)P.xbf16;
        auto ld = [&](int i) {
            const bl_v4i v = x[i];
            return make_uint4((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]);
        };
        float mx = 0.0f;
        for (int u = tid; u < groups; u += 256)
            mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(ld(2 * u)), bl_absmax8_bf16(ld(2 * u + 1))));
        mx = bl_wave_max(mx);
        if (lane == 0) fs[w] = mx;
        __syncthreads();
        const float gamma = fmaxf(fmaxf(fs[0], fs[1]), fmaxf(fs[2], fs[3]));
        const float gg = fmaxf(gamma, 1e-5f);
        const float inv = bl_div_rn(127.0f, gg);
        for (int u = tid; u < groups; u += 256) {
            uint32_t a0, a1, a2, a3;
            bl_quant8_words(ld(2 * u), inv, a0, a1);
            bl_quant8_words(ld(2 * u + 1), inv, a2, a3);
            part += bl_sum16(a0, a1, a2, a3);
            const bl_v4i qv = {(int)a0, (int)a1, (int)a2, (int)a3};
            if (owner && P.q_out) *(bl_gv4i*)(P.q_out + u * 16) = qv;
            bl_lds_put16(Qs, u, P.layout, a0, a1, a2, a3);
        }
        if (tid == 0) {
            const float sc = bl_div_rn(gg, 127.0f);
            misc[1] = __float_as_int(P.fixed_scale > 0.0f ? P.fixed_scale : sc);
            if (owner && P.scale_out) *(float BL_G*)P.scale_out = sc;
        }
        part = bl_wave_sum(part);
        if (lane == 0) ssum[w] = part;
        __syncthreads();
        if (tid == 0) misc[0] = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
    } else {
        const bl_gv4i* qg = (const bl_gv4i*)P.q;
        for (int u = tid; u < groups; u += 256) {
            const bl_v4i v = qg[u];
            bl_lds_put16(Qs, u, P.layout, (uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]);
        }
        if (tid == 0) {
            misc[0] = *(const int32_t BL_G*)P.rowsum;
            misc[1] = P.scale ? __float_as_int(*(const float BL_G*)P.scale) : 0;
        }
    }
    __syncthreads();
}

/* One product slice [ub, ue) of row groups, for a product whose lanes hold LP 16-byte weight
 * loads per row (k chunks g, g+G, .. of the row; G = 1 << lgG lanes per row, R = 64 / G rows
 * per wave-wide load).  A "unit" is S consecutive row groups: S*LP loads per lane per register
 * set.  The four waves of the workgroup take units round-robin.  Every load of the steady loop
 * is unconditional (out-of-range lanes read a clamped, valid address and meet the all-zero
 * chunk, or are never stored), so the hardware counter waits are exact and the loads of unit
 * i+1 stay in flight during the dot products of unit i.  The residual value of a row travels
 * with the row's weights: a load issued later, in the epilogue, could only be waited for
 * together with every weight load issued before it (with no residual every lane reads beta
 * instead, a valid address, and the value is not used). */
template <int LP, int S>
__device__ __forceinline__ void bl_stream_slice(const bl_stream_item& P, const int ub, const int ue,
                                                    int* __restrict__ Qs, int* __restrict__ misc,
                                                    const bool restage) {
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int N = P.N, nchunks = P.nchunks, lgG = P.lgG;
    const int R = 64 >> lgG;
    const int r = lane >> lgG, g = lane & ((1 << lgG) - 1);
    const int nunits = (ue - ub + S - 1) / S;            /* the last unit may be partial */
    const bl_gv4i* const wbase = (const bl_gv4i*)P.packed;
    int32_t BL_G* const acc_g = (int32_t BL_G*)P.acc;
    float BL_G* const y_g = (float BL_G*)P.y;
    const float BL_G* const res_g = (const float BL_G*)P.residual;
    const float BL_G* const res_base = res_g ? res_g : (const float BL_G*)P.beta;
    int coff[LP], qoff[LP];                              /* clamped k chunk of each load; its LDS image */
#pragma unroll
    for (int i = 0; i < LP; ++i) {
        const int chunk = g + (i << lgG);
        coff[i] = chunk < nchunks ? chunk : nchunks - 1;
        qoff[i] = (chunk < nchunks ? chunk : nchunks) * BL_QSTRIDE;   /* clamped lanes meet the zero chunk */
    }
    auto issue = [&](bl_v4i* p, float* rv, int unit) {
#pragma unroll
        for (int j = 0; j < S; ++j) {
            int n = (ub + unit * S + j) * R + r;
            n = n < N ? n : N - 1;
            const bl_gv4i* wrow = wbase + (int64_t)n * nchunks;
#pragma unroll
            for (int i = 0; i < LP; ++i) p[j * LP + i] = __builtin_nontemporal_load(wrow + coff[i]);
            rv[j] = res_base[res_g ? n : 0];
        }
    };
    bl_v4i pa[S * LP], pb[S * LP];
    float ra[S], rb[S];
    int u = w;                                           /* this wave's unit */
    if (u < nunits) issue(pa, ra, u);                    /* in flight during the staging */
    if (restage) __syncthreads();                        /* every wave is done with the previous image */
    bl_stream_stage(P, Qs, misc, ub == 0);
    if (u >= nunits) return;
    const int rs = misc[0];
    float cf = 0.0f;
    if (y_g) cf = *(const float BL_G*)P.beta * __int_as_float(misc[1]);

    auto finish = [&](const bl_v4i* p, const float* rv, int unit) {
#pragma unroll
        for (int j = 0; j < S; ++j) {
            int A[4] = {0, 0, 0, 0};
            /* The image does not change inside the loop, so the compiler would hoist these reads
             * out of it and hold them in 16 * LP registers again: the address is hidden from it. */
            bl_v4i a[1][4];
            auto rd = [&](int i, bl_v4i* dst) {
                int qo = qoff[i];
                asm volatile("" : "+v"(qo));
#pragma unroll
                for (int s = 0; s < 4; ++s) dst[s] = *(const bl_v4i*)(Qs + qo + s * 4);
            };
#pragma unroll
            for (int i = 0; i < LP; ++i) {
                rd(i, a[0]);
                bl_stream_dot(p[j * LP + i], a[0], A);
            }
            int v = A[0] + (A[1] >> 2) + ((A[2] + A[3]) >> 4);
            v = bl_group_sum_rt(v, lgG);
            const int rg = ub + unit * S + j;
            const int n = rg * R + r;
            if (g == 0 && rg < ue && n < N) {
                const int val = v - rs;
                if (acc_g) acc_g[n] = val;
                if (y_g) {
                    const float t = (float)val * cf;
                    y_g[n] = res_g ? rv[j] + t : t;
                }
            }
        }
    };
    for (;;) {
        if (u + 4 >= nunits) { finish(pa, ra, u); break; }
        issue(pb, rb, u + 4);
        finish(pa, ra, u);
        u += 4;
        if (u + 4 >= nunits) { finish(pb, rb, u); break; }
        issue(pa, ra, u + 4);
        finish(pb, rb, u);
        u += 4;
    }
}

/* ---- five weights per byte (BL_LAYOUT_TRIT5) ---------------------------------------------------
 * A byte b = ceil(v * 256 / 243) holds v = sum_i c_i * 3^(4-i), five offset codes c_i in {0,1,2}.
 * Multiplying by 3 moves the leading base-3 digit into bits 8..9 and leaves the rest of the
 * number in the low byte: five multiply-and-mask steps give the five digits, no table and no
 * division.  The four bytes of a word are handled as two pairs in 16-bit lanes (a byte times 3
 * fits 10 bits), and a byte permute gathers the four digits of step i into one register whose
 * bytes pair with k = 20*word + 4*i + 0..3: an operand of v_dot4_i32_i8 against the activations
 * in their natural order.  Per 16-byte load: 80 weights, 20 dot products, ~100 more vector
 * instructions: three times the work per weight of the 2-bit form. */
#define BL_T5_QSTRIDE 24      /* dwords per 80-weight chunk in LDS: 20 + 4 of padding */

__device__ __forceinline__ int bl_t5_dot(const bl_v4i p, const bl_v4i* a, int A) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t w = (uint32_t)p[d];
        uint32_t e = w & 0x00FF00FFu, o = (w >> 8) & 0x00FF00FFu;
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            e = (e << 1) + e;
            o = (o << 1) + o;
            const uint32_t dg = __builtin_amdgcn_perm(o, e, 0x07030501u);   /* bits 8..15 of the four lanes */
            A = __builtin_amdgcn_sdot4((int)dg, a[(5 * d + i) >> 2][(5 * d + i) & 3], A, false);
            if (i < 4) {
                e &= 0x00FF00FFu;
                o &= 0x00FF00FFu;
            }
        }
    }
    return A;
}

/* Stages the activation row for the five-per-byte form: the int8 row in its natural order, 80
 * bytes per chunk, zeros from the end of the row to the end of the last chunk and one all-zero
 * chunk behind it.  misc as in bl_stream_stage.  Ends with a barrier. */
__device__ __forceinline__ void bl_stream_stage_t5(const bl_stream_item& P, int* __restrict__ Qs,
                                                       int* __restrict__ misc, bool owner) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int groups = P.qgroups;
    float* fs = (float*)(misc + 2);
    int* ssum = misc + 6;
    auto put = [&](int u, bl_v4i v) { *(bl_v4i*)(Qs + (u / 5) * BL_T5_QSTRIDE + (u % 5) * 4) = v; };
    for (int u = groups + tid; u < (P.nchunks + 1) * 5; u += 256) put(u, bl_v4i{0, 0, 0, 0});
    int part = 0;
    if (P.xbf16) {
        const bl_gv4i* x = (const bl_gv4i*)P.xbf16;
        auto ld = [&](int i) {
            const bl_v4i v = x[i];
            return make_uint4((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]);
        };
        float mx = 0.0f;
        for (int u = tid; u < groups; u += 256)
            mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(ld(2 * u)), bl_absmax8_bf16(ld(2 * u + 1))));
        mx = bl_wave_max(mx);
        if (lane == 0) fs[w] = mx;
        __syncthreads();
        const float gamma = fmaxf(fmaxf(fs[0], fs[1]), fmaxf(fs[2], fs[3]));
        const float gg = fmaxf(gamma, 1e-5f);
        const float inv = bl_div_rn(127.0f, gg);
        for (int u = tid; u < groups; u += 256) {
            uint32_t a0, a1, a2, a3;
            bl_quant8_words(ld(2 * u), inv, a0, a1);
            bl_quant8_words(ld(2 * u + 1), inv, a2, a3);
            part += bl_sum16(a0, a1, a2, a3);
            const bl_v4i qv = {(int)a0, (int)a1, (int)a2, (int)a3};
            if (owner && P.q_out) *(bl_gv4i*)(P.q_out + u * 16) = qv;
            put(u, qv);
        }
        if (tid == 0) {
            const float sc = bl_div_rn(gg, 127.0f);
            misc[1] = __float_as_int(P.fixed_scale > 0.0f ? P.fixed_scale : sc);
            if (owner && P.scale_out) *(float BL_G*)P.scale_out = sc;
        }
        part = bl_wave_sum(part);
        if (lane == 0) ssum[w] = part;
        __syncthreads();
        if (tid == 0) misc[0] = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
    } else {
        const bl_gv4i* qg = (const bl_gv4i*)P.q;
        for (int u = tid; u < groups; u += 256) put(u, qg[u]);
        if (tid == 0) {
            misc[0] = *(const int32_t BL_G*)P.rowsum;
            misc[1] = P.scale ? __float_as_int(*(const float BL_G*)P.scale) : 0;
        }
    }
    __syncthreads();
}

/* bl_stream_slice for the five-per-byte form: the same double-buffered, unconditional loads; a
 * load is 80 weights against 20 activation dwords read from LDS right before its dot products. */
template <int LP>
__device__ __forceinline__ void bl_stream_slice_t5(const bl_stream_item& P, const int ub, const int ue,
                                                       int* __restrict__ Qs, int* __restrict__ misc,
                                                       const bool restage) {
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int N = P.N, nchunks = P.nchunks, lgG = P.lgG;
    const int R = 64 >> lgG;
    const int r = lane >> lgG, g = lane & ((1 << lgG) - 1);
    const int nunits = ue - ub;
    const bl_gv4i* const wbase = (const bl_gv4i*)P.packed;
    int32_t BL_G* const acc_g = (int32_t BL_G*)P.acc;
    float BL_G* const y_g = (float BL_G*)P.y;
    const float BL_G* const res_g = (const float BL_G*)P.residual;
    const float BL_G* const res_base = res_g ? res_g : (const float BL_G*)P.beta;
    int coff[LP], qoff[LP];
#pragma unroll
    for (int i = 0; i < LP; ++i) {
        const int chunk = g + (i << lgG);
        coff[i] = chunk < nchunks ? chunk : nchunks - 1;
        qoff[i] = (chunk < nchunks ? chunk : nchunks) * BL_T5_QSTRIDE;
    }
    auto issue = [&](bl_v4i* p, float& rv, int unit) {
        int n = (ub + unit) * R + r;
        n = n < N ? n : N - 1;
        const bl_gv4i* wrow = wbase + (int64_t)n * nchunks;
#pragma unroll
        for (int i = 0; i < LP; ++i) p[i] = __builtin_nontemporal_load(wrow + coff[i]);
        rv = res_base[res_g ? n : 0];
    };
    bl_v4i pa[LP], pb[LP];
    float ra = 0.0f, rb = 0.0f;
    int u = w;
    if (u < nunits) issue(pa, ra, u);
    if (restage) __syncthreads();
    bl_stream_stage_t5(P, Qs, misc, ub == 0);
    if (u >= nunits) return;
    const int rs = misc[0];
    float cf = 0.0f;
    if (y_g) cf = *(const float BL_G*)P.beta * __int_as_float(misc[1]);

    auto finish = [&](const bl_v4i* p, const float rv, int unit) {
        int A = 0;
#pragma unroll
        for (int i = 0; i < LP; ++i) {
            int qo = qoff[i];
            asm volatile("" : "+v"(qo));          /* keeps the reads inside the loop (see bl_stream_slice) */
            bl_v4i a[5];
#pragma unroll
            for (int t = 0; t < 5; ++t) a[t] = *(const bl_v4i*)(Qs + qo + t * 4);
            A = bl_t5_dot(p[i], a, A);
        }
        const int v = bl_group_sum_rt(A, lgG);
        const int rg = ub + unit;
        const int n = rg * R + r;
        if (g == 0 && n < N) {
            const int val = v - rs;
            if (acc_g) acc_g[n] = val;
            if (y_g) {
                const float t = (float)val * cf;
                y_g[n] = res_g ? rv + t : t;
            }
        }
    };
    for (;;) {
        if (u + 4 >= nunits) { finish(pa, ra, u); break; }
        issue(pb, rb, u + 4);
        finish(pa, ra, u);
        u += 4;
        if (u + 4 >= nunits) { finish(pb, rb, u); break; }
        issue(pa, ra, u + 4);
        finish(pb, rb, u);
        u += 4;
    }
}

/* Persistent grid: workgroup b walks the table slice wgstart[b] .. wgstart[b+1], each entry
 * (product, row group).  Two loop shapes cover every product: five loads per lane and row, and
 * up to four (a product with fewer leaves slots idle: clamped loads that hit the cache, the
 * all-zero chunk).  Four waves per SIMD, no scratch memory: a version that spilled lost a third
 * of the stream rate. */
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
void bl_stream_m1(const bl_stream_item* __restrict__ items, const int2* __restrict__ wgstart, const int q_ints) {
    extern __shared__ int lds[];                         /* q_ints ints of image + 16 */
    int* Qs = lds;
    int* misc = lds + q_ints;
    const int2 s0 = wgstart[blockIdx.x], s1 = wgstart[blockIdx.x + 1];
    const int p_first = __builtin_amdgcn_readfirstlane(s0.x), u_first = __builtin_amdgcn_readfirstlane(s0.y);
    const int p_last = __builtin_amdgcn_readfirstlane(s1.x), u_last = __builtin_amdgcn_readfirstlane(s1.y);
    bool staged = false;
    for (int pi = p_first; pi <= p_last; ++pi) {
        if (pi == p_last && u_last == 0) break;
        const bl_stream_item P = items[pi];
        const int ub = pi == p_first ? u_first : 0;
        const int ue = pi == p_last ? u_last : P.units;
        if (ub >= ue) continue;
        if (P.lp == 5) bl_stream_slice<5, 1>(P, ub, ue, Qs, misc, staged);
        else bl_stream_slice<4, 1>(P, ub, ue, Qs, misc, staged);
        staged = true;
    }
}

/* The same walk for a table in the five-per-byte form. */
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
void bl_stream_m1_t5(const bl_stream_item* __restrict__ items, const int2* __restrict__ wgstart, const int q_ints) {
    extern __shared__ int lds[];
    int* Qs = lds;
    int* misc = lds + q_ints;
    const int2 s0 = wgstart[blockIdx.x], s1 = wgstart[blockIdx.x + 1];
    const int p_first = __builtin_amdgcn_readfirstlane(s0.x), u_first = __builtin_amdgcn_readfirstlane(s0.y);
    const int p_last = __builtin_amdgcn_readfirstlane(s1.x), u_last = __builtin_amdgcn_readfirstlane(s1.y);
    bool staged = false;
    for (int pi = p_first; pi <= p_last; ++pi) {
        if (pi == p_last && u_last == 0) break;
        const bl_stream_item P = items[pi];
        const int ub = pi == p_first ? u_first : 0;
        const int ue = pi == p_last ? u_last : P.units;
        if (ub >= ue) continue;
        if (P.lp == 5) bl_stream_slice_t5<5>(P, ub, ue, Qs, misc, staged);
        else bl_stream_slice_t5<4>(P, ub, ue, Qs, misc, staged);
        staged = true;
    }
}

/* ---- k-major form (BL_LAYOUT_KMAJOR): skipping the weights of zero activations -----------------
 * Section 2 of the report takes squared ReLU in the feed-forward block for the sparsity it gives
 * the activations of the down projection.  Stored k-major (one row of N codes per input feature k),
 * the weights of a zero activation are simply not read.  A wave takes 64 consecutive k, finds the
 * non-zero activations with one ballot and walks them four at a time: lane l loads its dword
 * (16 output features) from each of the four rows, a byte permute puts the same byte of the four
 * rows side by side, and the mask-only level trick of the other kernels turns that into operands
 * of v_dot4_i32_i8 against the four activations (uniform, so they sit in a scalar register).
 * Every workgroup holds partial sums over its own k range: they meet in LDS, then in an int32
 * array in device memory (integer atomics: exact, order-free), and a small finishing kernel
 * subtracts the row sum, rescales, adds the residual and clears the array for the next run. */
template <int CB>
__device__ __forceinline__ void bl_km_slice(const bl_stream_item& P, const int ub, const int ue,
                                                int* __restrict__ Qs, int* __restrict__ misc,
                                                int* __restrict__ red, const bool restage) {
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ncols = P.nchunks, N = P.N;
    const uint32_t BL_G* const wbase = (const uint32_t BL_G*)P.packed;
    int col[CB];
    bool ok[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j) {
        const int c = 64 * j + lane;
        ok[j] = c < ncols;
        col[j] = ok[j] ? c : ncols - 1;
    }
    if (restage) __syncthreads();
    /* the int8 row in its natural order, zeros up to the end of the last 64-wide k block */
    {
        const int groups = P.qgroups, lw = tid >> 6;
        float* fs = (float*)(misc + 2);
        int* ssum = misc + 6;
        bl_v4i* Q4 = (bl_v4i*)Qs;
        for (int u = groups + tid; u < P.units * 4; u += 256) Q4[u] = bl_v4i{0, 0, 0, 0};
        for (int n = tid; n < ncols * 16; n += 256) red[n] = 0;
        if (P.xbf16) {
            const bl_gv4i* x = (const bl_gv4i*)P.xbf16;
            auto ld = [&](int i) {
                const bl_v4i v = x[i];
                return make_uint4((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]);
            };
            float mx = 0.0f;
            for (int u = tid; u < groups; u += 256)
                mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(ld(2 * u)), bl_absmax8_bf16(ld(2 * u + 1))));
            mx = bl_wave_max(mx);
            if (lane == 0) fs[lw] = mx;
            __syncthreads();
            const float gamma = fmaxf(fmaxf(fs[0], fs[1]), fmaxf(fs[2], fs[3]));
            const float gg = fmaxf(gamma, 1e-5f);
            const float inv = bl_div_rn(127.0f, gg);
            int part = 0;
            for (int u = tid; u < groups; u += 256) {
                uint32_t a0, a1, a2, a3;
                bl_quant8_words(ld(2 * u), inv, a0, a1);
                bl_quant8_words(ld(2 * u + 1), inv, a2, a3);
                part += bl_sum16(a0, a1, a2, a3);
                const bl_v4i qv = {(int)a0, (int)a1, (int)a2, (int)a3};
                if (ub == 0 && P.q_out) *(bl_gv4i*)(P.q_out + u * 16) = qv;
                Q4[u] = qv;
            }
            part = bl_wave_sum(part);
            if (lane == 0) ssum[lw] = part;
            __syncthreads();
            if (tid == 0 && ub == 0) {
                const float sc = bl_div_rn(gg, 127.0f);
                *(int32_t BL_G*)P.rowsum_pub = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
                *(float BL_G*)P.scale_pub = P.fixed_scale > 0.0f ? P.fixed_scale : sc;
                if (P.scale_out) *(float BL_G*)P.scale_out = sc;
            }
        } else {
            const bl_gv4i* qg = (const bl_gv4i*)P.q;
            for (int u = tid; u < groups; u += 256) Q4[u] = qg[u];
        }
        __syncthreads();
    }
    int A[CB][4][4];
#pragma unroll
    for (int j = 0; j < CB; ++j)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t) A[j][b][t] = 0;

    /* the stream of (four non-zero activations, their weight dwords): one step ahead of the arithmetic */
    int u = ub + w, k0 = 0, qv = 0;
    uint64_t mask = 0;
    auto fetch = [&](uint32_t (*wv)[4], int& q4) -> bool {
        while (mask == 0 && u < ue) {
            k0 = u * 64;
            qv = (int)((const int8_t*)Qs)[k0 + lane];
            mask = __ballot(qv != 0);
            u += 4;
        }
        if (mask == 0) return false;
        int kk[4];
        uint32_t q = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (mask) {
                const int idx = __builtin_amdgcn_readfirstlane(__builtin_ctzll(mask));
                mask &= mask - 1;
                kk[i] = idx;
                q |= ((uint32_t)__builtin_amdgcn_readlane(qv, idx) & 0xFFu) << (8 * i);
            } else {
                kk[i] = kk[0];                    /* a valid row; its activation byte stays 0 */
            }
        }
        q4 = (int)q;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t BL_G* row = wbase + (int64_t)(k0 + kk[i]) * ncols;
#pragma unroll
            for (int j = 0; j < CB; ++j) wv[j][i] = __builtin_nontemporal_load(row + col[j]);
        }
        return true;
    };
    auto compute = [&](const uint32_t (*wv)[4], const int q4) {
#pragma unroll
        for (int j = 0; j < CB; ++j)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                /* byte b of the four rows side by side: byte i of R = codes of (k_i, n = 16c + 4b + 0..3) */
                const uint32_t sel = 0x0C0C0400u + 0x0101u * (uint32_t)b;         /* [s1.b, s0.b, 0, 0] */
                const uint32_t lo = __builtin_amdgcn_perm(wv[j][1], wv[j][0], sel);
                const uint32_t hi = __builtin_amdgcn_perm(wv[j][3], wv[j][2], sel);
                const uint32_t R = lo | (hi << 16);
                A[j][b][0] = __builtin_amdgcn_sdot4((int)(R & 0x03030303u), q4, A[j][b][0], false);
                A[j][b][1] = __builtin_amdgcn_sdot4((int)(R & 0x0C0C0C0Cu), q4, A[j][b][1], false);
                A[j][b][2] = __builtin_amdgcn_sdot4((int)(R & 0x30303030u), q4, A[j][b][2], false);
                A[j][b][3] = __builtin_amdgcn_sdot4((int)((R >> 2) & 0x30303030u), q4, A[j][b][3], false);
            }
    };
    uint32_t wa[CB][4], wb[CB][4];
    int qa = 0, qb = 0;
    bool have = fetch(wa, qa);
    while (have) {
        const bool have2 = fetch(wb, qb);
        compute(wa, qa);
        if (!have2) break;
        have = fetch(wa, qa);
        compute(wb, qb);
    }
    /* partial sums of the four waves meet in LDS, then go to the product's int32 array */
#pragma unroll
    for (int j = 0; j < CB; ++j)
        if (ok[j]) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int n0 = 16 * (64 * j + lane) + 4 * b;
                const int v0 = A[j][b][0], v1 = A[j][b][1] >> 2, v2 = A[j][b][2] >> 4, v3 = A[j][b][3] >> 4;
                if (v0) atomicAdd(red + n0, v0);
                if (v1) atomicAdd(red + n0 + 1, v1);
                if (v2) atomicAdd(red + n0 + 2, v2);
                if (v3) atomicAdd(red + n0 + 3, v3);
            }
        }
    __syncthreads();
    for (int n = tid; n < N; n += 256) {
        const int v = red[n];
        if (v) atomicAdd((int32_t*)P.acc_ws + n, v);
    }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
void bl_stream_m1_km(const bl_stream_item* __restrict__ items, const int2* __restrict__ wgstart, const int q_ints,
                     const int red_ints) {
    extern __shared__ int lds[];
    int* Qs = lds;
    int* red = lds + q_ints;
    int* misc = red + red_ints;
    const int2 s0 = wgstart[blockIdx.x], s1 = wgstart[blockIdx.x + 1];
    const int p_first = __builtin_amdgcn_readfirstlane(s0.x), u_first = __builtin_amdgcn_readfirstlane(s0.y);
    const int p_last = __builtin_amdgcn_readfirstlane(s1.x), u_last = __builtin_amdgcn_readfirstlane(s1.y);
    bool staged = false;
    for (int pi = p_first; pi <= p_last; ++pi) {
        if (pi == p_last && u_last == 0) break;
        const bl_stream_item P = items[pi];
        const int ub = pi == p_first ? u_first : 0;
        const int ue = pi == p_last ? u_last : P.units;
        if (ub >= ue) continue;
        switch (P.lp) {
            case 1: bl_km_slice<1>(P, ub, ue, Qs, misc, red, staged); break;
            case 2: bl_km_slice<2>(P, ub, ue, Qs, misc, red, staged); break;
            default: bl_km_slice<3>(P, ub, ue, Qs, misc, red, staged); break;
        }
        staged = true;
    }
}

/* Finishing kernel of the k-major form: grid (ceil(max N / 256), products). */
__global__ __launch_bounds__(256) void bl_km_finish(const bl_stream_item* __restrict__ items) {
    const bl_stream_item& P = items[blockIdx.y];
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= P.N) return;
    const int val = P.acc_ws[n] - *P.rowsum_fin;
    P.acc_ws[n] = 0;
    if (P.acc) P.acc[n] = val;
    if (P.y) {
        const float cf = *P.beta * *P.scale_fin;
        const float t = (float)val * cf;
        P.y[n] = P.residual ? P.residual[n] + t : t;
    }
}


/* ---- batched form: 2..64 tokens per table entry on the matrix cores --------------------------
 * The same persistent walk for a few tokens per product (batched decode: the packed weights are
 * still read once, Section 5.1).  Workgroups of eight waves.  The int8 activations of all m
 * tokens of the product live in LDS for the workgroup (m rows of Kp + 16 bytes: the 16 spread
 * the rows over the banks), staged once per product and workgroup, so between two products no
 * wave waits for another: a wave takes row groups of 32 weight rows round-robin and streams
 * their packed bytes global -> registers in batches of 32 rows x 512 k (4 KiB: four wave-wide
 * loads in which eight consecutive lanes fetch 128 consecutive bytes of one row, the access
 * pattern of the one-token kernel), two batches in flight while a third is multiplied.
 * The matrix core wants another lane order (lane r + 32h supplies sixteen consecutive k of row
 * r), so a landed batch takes one trip through a 4 KiB tile of LDS that belongs to the wave
 * alone (ds_write_b128 as loaded, ds_read_b128 as needed; 16-byte items XOR-swizzled against
 * the row so that both directions are free of bank conflicts; a wave's LDS operations execute
 * in order, so no barrier is involved).  Each 16-byte item is four packed words; a word is
 * opened into sixteen int8 codes by shift and mask and is the B operand of one
 * v_mfma_i32_32x32x32_i8 (two for more than 32 tokens) whose A operand is the same sixteen k of
 * token r (and 32 + r) read from the image
 * (any k order serves as long as both operands agree).  Lanes whose chunk lies behind the row's
 * end re-read its last chunk and meet sixteen zero bytes kept behind the image; tokens behind
 * m re-read token m-1 and are never stored.  Offset codes: sum_k q of the token is subtracted
 * once per output. */
#define BL_MB_THREADS 512
#define BL_MB_WAVES 8
#define BL_MB_MISC 576        /* bytes behind the image: 64 zero bytes, 64 row sums, 64 factors */
#define BL_MB_TILE 4096       /* bytes of a wave's private tile */

template <int TB, bool RES>
__device__ __forceinline__ void bl_stream_slice_mb(const bl_stream_item& P, const int ub, const int ue,
                                                   uint8_t* __restrict__ img, uint8_t* __restrict__ tiles,
                                                   const bool restage) {
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5, r8 = lane >> 3, c8 = lane & 7;
    const int N = P.N, nchunks = P.nchunks, m = P.m, rowc = P.row_chunks, c0 = P.c0;
    const int stride = nchunks * 64 + 16;                               /* image row: the entry's k part + 16 */
    const int nb = (nchunks + 7) / 8;                                   /* batches of 512 k per row */
    int32_t BL_G* const ws_g = (int32_t BL_G*)P.acc_ws;                 /* k parts of a split product meet here */
    const bl_gv4i* const wbase = (const bl_gv4i*)P.packed;
    int32_t BL_G* const acc_g = (int32_t BL_G*)P.acc;
    float BL_G* const y_g = (float BL_G*)P.y;
    const float BL_G* const res_g = (const float BL_G*)P.residual;
    uint8_t* const zero = img + m * stride;                             /* 64 zero bytes */
    int* const rs_s = (int*)(zero + 64);
    float* const cf_s = (float*)(rs_s + 64);
    bl_v4i* const tile = (bl_v4i*)(tiles + w * BL_MB_TILE);

    /* batch b of row group rg: load i covers rows 8i .. 8i+7, lane (r8, c8) chunk 8b + c8 of row 8i + r8 */
    auto issue = [&](bl_v4i* p, int rg, int b) {
        const int chunk = b * 8 + c8;
        const int cc = chunk < nchunks ? chunk : nchunks - 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int n = rg * 32 + i * 8 + r8;
            n = n < N ? n : N - 1;
            p[i] = __builtin_nontemporal_load(wbase + (int64_t)n * rowc + c0 + cc);
        }
    };
    int arow[TB];                                                        /* token l32 of tile tt (clamped) */
#pragma unroll
    for (int tt = 0; tt < TB; ++tt) arow[tt] = (tt * 32 + l32 < m ? tt * 32 + l32 : m - 1) * stride;
    const int zoff = m * stride;
    auto process = [&](const bl_v4i* p, int b, bl_v16i* C) {
        /* registers -> tile: row 8i + r8, item c8 ^ ((row / 2) % 8) */
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[(i * 8 + r8) * 8 + (c8 ^ (((i * 8 + r8) >> 1) & 7))] = p[i];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bl_v4i w4 = tile[l32 * 8 + ((2 * j + h) ^ ((l32 >> 1) & 7))];
            const int chunk = b * 8 + 2 * j + h;
            const bool valid = chunk < nchunks;
            int ao[TB];
#pragma unroll
            for (int tt = 0; tt < TB; ++tt) {
                ao[tt] = valid ? arow[tt] + chunk * 64 : zoff;
                asm volatile("" : "+v"(ao[tt]));                        /* read at the point of use, not hoisted */
            }
            const int step = valid ? 16 : 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t wd = (uint32_t)w4[t];
                const uint32_t l0 = wd & 0x03030303u, l1 = (wd >> 2) & 0x03030303u, l2 = (wd >> 4) & 0x03030303u,
                               l3 = (wd >> 6) & 0x03030303u;
                const bl_v4i bop = {(int)l0, (int)l1, (int)l2, (int)l3};
#pragma unroll
                for (int tt = 0; tt < TB; ++tt) {
                    const bl_v4i a = *(const bl_v4i*)(img + ao[tt] + t * step);
                    C[tt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, bop, C[tt], 0, 0, 0);
                }
            }
        }
    };
    /* lane (n = l32, h) holds, in element v of tile tt, token 32tt + (v/4)*8 + 4h + v%4 of output feature n */
    auto epilogue = [&](bl_v16i& C, int rg, int tt) {
        bl_mfma_fence();
        /* (the row length and the lane half are hidden from the compiler here: it would otherwise
         * keep the sixteen 64-bit row offsets of a lane's tokens in registers across the k loop) */
        int Nl = N, hl = h;
        asm volatile("" : "+s"(Nl));
        asm volatile("" : "+v"(hl));
        const int n = rg * 32 + l32;
        const bool nok = n < N;
        float rv[16];
        if (RES) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = tt * 32 + (v >> 2) * 8 + hl * 4 + (v & 3);
                rv[v] = (nok && t < m) ? res_g[(int64_t)t * Nl + n] : 0.0f;
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int t = tt * 32 + (v >> 2) * 8 + hl * 4 + (v & 3);
            if (nok && t < m) {
                if (ws_g) {                                             /* one k part: integer atomics, exact and order-free */
                    atomicAdd((int*)(ws_g + (int64_t)t * Nl + n), C[v]);
                    continue;
                }
                const int val = C[v] - rs_s[t];
                if (acc_g) acc_g[(int64_t)t * Nl + n] = val;
                if (y_g) {
                    const float o = (float)val * cf_s[t];
                    y_g[(int64_t)t * Nl + n] = RES ? rv[v] + o : o;
                }
            }
        }
    };

    bl_v4i pa[4], pb[4], pc[4];
    const int rg0 = ub + w;
    const bool work = rg0 < ue;
    /* issue cursor (two batches ahead of the process cursor); behind the wave's last row group it
     * stays on that row group: valid addresses, data never used */
    int irg = rg0, ib = 0;
    auto advance = [&]() {
        if (++ib == nb) {
            ib = 0;
            if (irg + BL_MB_WAVES < ue) irg += BL_MB_WAVES;
        }
    };
    if (work) {                                                          /* in flight during the staging */
        issue(pa, irg, ib);
        advance();
        issue(pb, irg, ib);
        advance();
    }
    if (restage) __syncthreads();                                       /* every wave is done with the previous image */
    {
        /* stage the m token rows (16 bytes per thread and step), the zero bytes and the token terms */
        const int upr = nchunks * 4, ldu = P.ldq / 16;
        const bl_gv4i* qg = (const bl_gv4i*)P.q + c0 * 4;
        for (int u = tid; u < m * upr; u += BL_MB_THREADS) {
            const int row = u / upr, c = u - row * upr;
            *(bl_v4i*)(img + row * stride + c * 16) = qg[row * ldu + c];
        }
        if (tid < 16) ((int*)zero)[tid] = 0;
        if (tid < 64) {
            const int t = tid < m ? tid : m - 1;
            rs_s[tid] = ((const int32_t BL_G*)P.rowsum)[t];
            cf_s[tid] = P.y ? *(const float BL_G*)P.beta * ((const float BL_G*)P.scale)[t] : 0.0f;
        }
    }
    __syncthreads();
    if (!work) return;

    int prg = rg0, pbt = 0;                                             /* process cursor */
    bl_v16i C[TB];
#pragma unroll
    for (int tt = 0; tt < TB; ++tt)
#pragma unroll
        for (int v = 0; v < 16; ++v) C[tt][v] = 0;
    /* one batch out of `buf`; true when the wave's last row group is finished */
    auto step = [&](const bl_v4i* buf) {
        process(buf, pbt, C);
        if (++pbt < nb) return false;
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) {
            epilogue(C[tt], prg, tt);
#pragma unroll
            for (int v = 0; v < 16; ++v) C[tt][v] = 0;
        }
        pbt = 0;
        prg += BL_MB_WAVES;
        return prg >= ue;
    };
    while (true) {
        issue(pc, irg, ib);
        advance();
        if (step(pa)) break;
        issue(pa, irg, ib);
        advance();
        if (step(pb)) break;
        issue(pb, irg, ib);
        advance();
        if (step(pc)) break;
    }
}

/* TB = token tiles of 32 an entry may hold: 1 for tables of at most 32 tokens (fewer registers:
 * two workgroups per compute unit when the images are small), 2 beyond. */
template <int TB>
__global__ __launch_bounds__(BL_MB_THREADS)
void bl_stream_mb(const bl_stream_item* __restrict__ items, const int2* __restrict__ wgstart) {
    extern __shared__ __attribute__((aligned(16))) uint8_t img[];   /* tiles of the eight waves, then the image */
    uint8_t* const tiles = img;
    uint8_t* const image = img + BL_MB_WAVES * BL_MB_TILE;
    const int2 s0 = wgstart[blockIdx.x], s1 = wgstart[blockIdx.x + 1];
    const int p_first = __builtin_amdgcn_readfirstlane(s0.x), u_first = __builtin_amdgcn_readfirstlane(s0.y);
    const int p_last = __builtin_amdgcn_readfirstlane(s1.x), u_last = __builtin_amdgcn_readfirstlane(s1.y);
    bool staged = false;
    for (int pi = p_first; pi <= p_last; ++pi) {
        if (pi == p_last && u_last == 0) break;
        const bl_stream_item P = items[pi];
        const int ub = pi == p_first ? u_first : 0;
        const int ue = pi == p_last ? u_last : P.units;
        if (ub >= ue) continue;
        if (TB == 2 && P.m > 32) {
            if (P.residual) bl_stream_slice_mb<TB, true>(P, ub, ue, image, tiles, staged);
            else bl_stream_slice_mb<TB, false>(P, ub, ue, image, tiles, staged);
        } else {
            if (P.residual) bl_stream_slice_mb<1, true>(P, ub, ue, image, tiles, staged);
            else bl_stream_slice_mb<1, false>(P, ub, ue, image, tiles, staged);
        }
        staged = true;
    }
}

/* Finishing kernel of the batched form for products that were split along k: subtracts the
 * row sum, rescales, adds the residual, stores, and clears the partial sums for the next run.
 * grid (ceil(max M*N / 1024), split products). */
struct bl_mb_fin_item {
    int32_t* ws;              /* [M][N] partial sums */
    const int32_t* rowsum;
    const float* scale;
    const float* beta;
    const float* residual;
    int32_t* acc;
    float* y;
    int M, N;
};
__global__ __launch_bounds__(256) void bl_mb_finish(const bl_mb_fin_item* __restrict__ items) {
    const bl_mb_fin_item F = items[blockIdx.y];
    const int64_t total = (int64_t)F.M * F.N;
    const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    if (base >= total) return;
    const float bt = F.y ? *F.beta : 0.0f;
    /* four elements per thread, every load of a step issued before the first use */
    int part[4], rs[4];
    float cf[4], res[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t e = base + j * 256;
        const bool ok = e < total;
        const int t = ok ? (int)(e / F.N) : 0;
        part[j] = ok ? F.ws[e] : 0;
        rs[j] = F.rowsum[t];
        cf[j] = F.y ? F.scale[t] : 0.0f;
        res[j] = (ok && F.residual) ? F.residual[e] : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t e = base + j * 256;
        if (e < total) {
            const int val = part[j] - rs[j];
            F.ws[e] = 0;
            if (F.acc) F.acc[e] = val;
            if (F.y) {
                const float o = (float)val * (bt * cf[j]);
                F.y[e] = F.residual ? res[j] + o : o;
            }
        }
    }
}

/* ---- host side ---------------------------------------------------------------------------- */

#define BL_STREAM_LMAX 5
#define BL_STREAM_MAX_BLOCKS 4096
#define BL_STREAM_LDS_BYTES                                                                          \
    (layout == BL_LAYOUT_KMAJOR ? max_units * 64 + max_cols * 64 + 64                                \
                                : (max_chunks + 1) * (layout == BL_LAYOUT_TRIT5 ? BL_T5_QSTRIDE : BL_QSTRIDE) * 4 + 64)
#define BL_KM_MAX_N 3072      /* k-major form: at most three dword columns of 64 lanes per weight row (48 sums per lane) */

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

/* Device buffer layout: [items][slice table][preparation items][rowsum_ws][scale_ws][q_ws][acc_ws]. */
struct bl_stream_layout {
    size_t wg_off, prep_off, rowsum_off, scale_off, q_off, acc_off, total;
};
static bl_stream_layout stream_layout(int count, size_t q_bytes, size_t acc_bytes = 0) {
    bl_stream_layout L;
    L.wg_off = align_up((size_t)count * sizeof(bl_stream_item), 256);
    L.prep_off = L.wg_off + align_up((size_t)(BL_STREAM_MAX_BLOCKS + 1) * sizeof(int2), 256);
    L.rowsum_off = L.prep_off + align_up((size_t)count * sizeof(bl_stream_prep_item), 256);
    L.scale_off = L.rowsum_off + align_up((size_t)count * 4, 256);
    L.q_off = L.scale_off + align_up((size_t)count * 4, 256);
    L.acc_off = L.q_off + align_up(q_bytes, 256);
    L.total = L.acc_off + align_up(acc_bytes, 256);
    return L;
}

/* Cuts a table of products (units[i] row groups of unit_cost[i] each, enter_cost[i] for every
 * workgroup that enters product i) into `blocks` contiguous slices of about equal cost: walk the
 * row groups once, cutting whenever a workgroup's cost reaches the target; the last workgroup
 * takes what is left.  Returns blocks + 1 positions (product, row group). */
static std::vector<int2> cut_slices(const std::vector<int>& units, const std::vector<int64_t>& unit_cost,
                                    const std::vector<int64_t>& enter_cost, int blocks) {
    const int count = (int)units.size();
    std::vector<int2> wg((size_t)blocks + 1);
    int64_t all = 0;
    for (int i = 0; i < count; ++i) all += (int64_t)units[(size_t)i] * unit_cost[(size_t)i] + enter_cost[(size_t)i];
    /* every cut inside a product adds one more entry, so the target is refined until the
     * last workgroup (which takes what is left) is no longer than the others */
    int64_t target = all / blocks + 1;
    for (int iter = 0; iter < 12; ++iter) {
        int pi = 0, unit = 0;
        for (int b = 0; b < blocks; ++b) {
            wg[(size_t)b] = make_int2(pi, unit);
            int64_t c = 0;
            bool entered = false;
            while (pi < count && b < blocks - 1) {
                if (!entered) { c += enter_cost[(size_t)pi]; entered = true; }
                const int64_t uc = unit_cost[(size_t)pi];
                const int64_t room = target - c;
                const int64_t take = room > 0 ? (room + uc - 1) / uc : 0;
                const int left = units[(size_t)pi] - unit;
                if (take >= left) {
                    c += (int64_t)left * uc;
                    ++pi;
                    unit = 0;
                    entered = false;
                    if (c >= target) break;
                } else {
                    unit += (int)take;
                    break;
                }
            }
        }
        /* cost of what is left for the last workgroup */
        int64_t last = 0;
        {
            int pi = wg[(size_t)blocks - 1].x, unit = wg[(size_t)blocks - 1].y;
            for (; pi < count; ++pi, unit = 0)
                if (units[(size_t)pi] > unit)
                    last += enter_cost[(size_t)pi] + (int64_t)(units[(size_t)pi] - unit) * unit_cost[(size_t)pi];
        }
        if (last <= target + target / 64) break;
        target += (last - target) / blocks + 1;
    }
    /* normalise an end position (count, 0) to (count - 1, units): the kernel never reads entry `count` */
    for (int b = 0; b <= blocks; ++b)
        if (b == blocks || wg[(size_t)b].x >= count) wg[(size_t)b] = make_int2(count - 1, units[(size_t)count - 1]);
    return wg;
}

static bool desc_is_fused(const bl_decode_desc& d) { return d.X || d.prod.in0; }

static bl_status check_stack_desc(const bl_decode_desc& d, int layout) {
    if (!d.packed || !d.beta) return BL_ERR_NULL;
    const bool fused = desc_is_fused(d);
    if (!fused && !d.q) return BL_ERR_NULL;
    if (!d.acc && !d.y) return BL_ERR_NULL;
    if (!fused && d.y && !d.scale) return BL_ERR_NULL;
    if (!bl_shape_ok(d.N, d.K) || d.K > 64 * 64 * BL_STREAM_LMAX || d.N > (1 << 28)) return BL_ERR_SHAPE;
    if (fused && d.K % 64 != 0) return BL_ERR_SHAPE;     /* bf16 / producer rows are read 16 elements at a time */
    if (layout == BL_LAYOUT_KMAJOR && d.N > BL_KM_MAX_N) return BL_ERR_SHAPE;
    if (layout < BL_LAYOUT_ROWMAJOR || layout > BL_LAYOUT_KMAJOR) return BL_ERR_LAYOUT;
    if (!bl_aligned(d.packed, 16) || !bl_aligned(d.X, 16) || !bl_aligned(d.q, 16) || !bl_aligned(d.q_out, 16) ||
        !bl_aligned(d.acc, 4) || !bl_aligned(d.y, 4) || !bl_aligned(d.scale, 4) || !bl_aligned(d.beta, 4) ||
        !bl_aligned(d.rowsum, 4) || !bl_aligned(d.scale_out, 4) || !bl_aligned(d.residual, 4))
        return BL_ERR_ALIGN;
    return BL_OK;
}

/* ---- batched form (2 .. BL_STACK_MAX_TOKENS tokens per product) ------------------------------ */

#define BL_MB_LDS_MAX (160 * 1024)

/* How one product is entered in the table: token groups of at most 64 (two matrix-core tiles),
 * the M tokens split evenly over the fewest groups, and k parts of whole 512-k batches so that a
 * group's rows of one part fit LDS beside each other.  A product with more than one k part
 * collects its partial sums in `ws` and is finished by bl_mb_finish. */
struct mb_split {
    int groups, per_group;    /* token groups, tokens per group (the last may hold fewer) */
    int parts, part_chunks;   /* k parts, 16-byte chunks per part (the last may hold fewer) */
};
static bool mb_split_product(int64_t M, int64_t Kp, mb_split* sp) {
    const int64_t budget = BL_MB_LDS_MAX - BL_MB_MISC - BL_MB_WAVES * BL_MB_TILE;
    const int64_t nchunks = Kp / 64;
    /* two matrix-core tiles of tokens per entry where their rows fit LDS whole (the weights are
     * then read once and nothing meets through atomics: measured at M = 64, 2560 <= K: two groups
     * of 32 tokens 267 us per 30 layers, one group of 64 in k parts 375 us); else one tile */
    sp->groups = (int)((M + 63) / 64);
    sp->per_group = (int)((M + sp->groups - 1) / sp->groups);
    if (sp->per_group > 32 && (int64_t)sp->per_group * (Kp + 16) > budget) {
        sp->groups = (int)((M + 31) / 32);
        sp->per_group = (int)((M + sp->groups - 1) / sp->groups);
    }
    int64_t parts = ((int64_t)sp->per_group * (Kp + 16) + budget - 1) / budget;
    int64_t pc = (nchunks + parts - 1) / parts;
    pc = (pc + 7) / 8 * 8;
    while (pc > 8 && (int64_t)sp->per_group * (pc * 64 + 16) > budget) pc -= 8;
    if ((int64_t)sp->per_group * (pc * 64 + 16) > budget) return false;
    sp->part_chunks = (int)pc;
    sp->parts = (int)((nchunks + pc - 1) / pc);
    return true;
}

/* Device buffer of the batched form: [entries][slice table][finishing items][partial sums]. */
struct mb_layout_t {
    size_t wg_off, fin_off, ws_off, total;
};
static mb_layout_t mb_layout(int64_t entries, int count, size_t ws_bytes) {
    mb_layout_t L;
    L.wg_off = align_up((size_t)entries * sizeof(bl_stream_item), 256);
    L.fin_off = L.wg_off + align_up((size_t)(BL_STREAM_MAX_BLOCKS + 1) * sizeof(int2), 256);
    L.ws_off = L.fin_off + align_up((size_t)count * sizeof(bl_mb_fin_item), 256);
    L.total = L.ws_off + align_up(ws_bytes, 256);
    return L;
}

static bl_status check_batched_desc(const bl_decode_desc& d, int layout) {
    if (!d.packed || !d.beta || !d.q || !d.rowsum) return BL_ERR_NULL;
    if (d.X || d.prod.in0) return BL_ERR_VALUE;            /* int8 inputs only: quantise with bl_quant_act_int8 */
    if (!d.acc && !d.y) return BL_ERR_NULL;
    if (d.y && !d.scale) return BL_ERR_NULL;
    if (!bl_shape_ok(d.N, d.K) || d.N > (1 << 24)) return BL_ERR_SHAPE;
    if (layout != BL_LAYOUT_K16) return BL_ERR_LAYOUT;
    if (!bl_aligned(d.packed, 16) || !bl_aligned(d.q, 16) || !bl_aligned(d.acc, 4) || !bl_aligned(d.y, 4) ||
        !bl_aligned(d.scale, 4) || !bl_aligned(d.beta, 4) || !bl_aligned(d.rowsum, 4) || !bl_aligned(d.residual, 4))
        return BL_ERR_ALIGN;
    return BL_OK;
}

static bool mb_sizes(const bl_decode_desc* descs, int count, int64_t M, int64_t* entries, size_t* ws_bytes) {
    *entries = 0;
    *ws_bytes = 0;
    for (int i = 0; i < count; ++i) {
        if (!bl_shape_ok(descs[i].N, descs[i].K) || descs[i].N > (1 << 24)) return false;
        mb_split sp;
        if (!mb_split_product(M, bl_kpad(descs[i].K), &sp)) return false;
        *entries += (int64_t)sp.groups * sp.parts;
        if (sp.parts > 1) *ws_bytes += align_up((size_t)(M * descs[i].N * 4), 256);
    }
    return *entries <= 64 * BL_STACK_MAX_COUNT;
}

static bool mb_tile_route(const bl_decode_desc* descs, int count, int64_t M);
static size_t tile_route_total(const bl_decode_desc* descs, int count);

extern "C" size_t bl_stack_table_bytes_batched(const bl_decode_desc* descs, int count, int64_t M) {
    if (!descs || count < 1 || count > BL_STACK_MAX_COUNT || M < 2 || M > BL_STACK_MAX_TOKENS) return 0;
    int64_t entries = 0;
    size_t ws_bytes = 0;
    if (!mb_sizes(descs, count, M, &entries, &ws_bytes)) return 0;
    size_t total = mb_layout(entries, count, ws_bytes).total;
    if (mb_tile_route(descs, count, M)) {
        const size_t tt = tile_route_total(descs, count);
        if (tt > total) total = tt;
    }
    return total;
}

/* More than 48 tokens per product: the token rows of most products no longer fit LDS whole, the
 * work is a dense contraction, and the table is walked by the prefill tile kernel instead
 * (64 x 128 tiles, both operands streamed through LDS per k step, weights read once; measured on
 * the 30-layer table at M = 64: 6.3 us per layer against 9.3 with two token groups of 32; at
 * M = 48 the two are equal, below the LDS-resident form wins).  Needs rows padded to 128. */
#define BL_MB_TILE_ROUTE_MIN 49
static bool mb_tile_route(const bl_decode_desc* descs, int count, int64_t M) {
    if (M < BL_MB_TILE_ROUTE_MIN) return false;
    int64_t tiles = 0;
    for (int i = 0; i < count; ++i) {
        if (bl_kpad(descs[i].K) % 128 != 0) return false;
        tiles += (descs[i].N + 127) / 128;
    }
    return tiles <= ((int64_t)1 << 22);       /* beyond ~4 M tiles (a 16 MB tile list) the table stays on bl_stream_mb */
}

/* Device buffer of the tile route: [products][first tile of each product][first list position of
 * each workgroup][tile list]. */
struct tile_layout_t {
    size_t t0_off, wg_off, list_off, total;
};
static tile_layout_t tile_layout(int count, int64_t tiles) {
    tile_layout_t L;
    L.t0_off = align_up((size_t)count * sizeof(bl_tile_item), 256);
    L.wg_off = L.t0_off + align_up((size_t)count * sizeof(int), 256);
    L.list_off = L.wg_off + align_up((size_t)(BL_STREAM_MAX_BLOCKS + 1) * sizeof(int), 256);
    L.total = L.list_off + align_up((size_t)tiles * sizeof(int), 256);
    return L;
}
static int64_t tile_route_tiles(const bl_decode_desc* descs, int count) {
    int64_t tiles = 0;
    for (int i = 0; i < count; ++i) tiles += (descs[i].N + 127) / 128;
    return tiles;
}

static size_t tile_route_total(const bl_decode_desc* descs, int count) {
    return tile_layout(count, tile_route_tiles(descs, count)).total;
}

static bl_status stack_build_tiles(const bl_decode_desc* descs, int count, int layout, int M, void* table,
                                   bl_stack_plan* plan, hipStream_t st) {
    const int resident = bl_gemm_table_blocks();
    if (resident < 1) return BL_ERR_HIP;
    const int64_t tiles = tile_route_tiles(descs, count);
    const tile_layout_t L = tile_layout(count, tiles);
    int blocks = (int)(tiles < resident ? tiles : resident);
    if (blocks > BL_STREAM_MAX_BLOCKS) blocks = BL_STREAM_MAX_BLOCKS;
    std::vector<uint8_t> blob(L.total, 0);
    bl_tile_item* items = (bl_tile_item*)blob.data();
    int* tile0 = (int*)(blob.data() + L.t0_off);
    int* wg_start = (int*)(blob.data() + L.wg_off);
    int* tile_list = (int*)(blob.data() + L.list_off);
    int64_t packed_bytes = 0, t = 0;
    /* (cost, first tile, tiles) of each product; cost of a tile = its k steps + a fixed part for
     * set-up and stores */
    std::vector<std::pair<int, int>> by_cost;             /* (-cost, product) */
    for (int i = 0; i < count; ++i) {
        const bl_decode_desc& d = descs[i];
        const int64_t Kp = bl_kpad(d.K);
        items[i] = bl_tile_item{d.packed, d.q, d.rowsum, d.beta, d.y ? d.scale : nullptr, d.residual, d.acc, d.y,
                                (int)d.N, (int)Kp};
        tile0[i] = (int)t;
        t += (d.N + 127) / 128;
        packed_bytes += d.N * (Kp / 4);
        by_cost.push_back({-(int)(Kp / 128 + 4), i});
    }
    /* longest tiles first, each to the workgroup with the least work so far */
    std::sort(by_cost.begin(), by_cost.end());
    std::vector<std::vector<int>> lists((size_t)blocks);
    std::priority_queue<std::pair<int64_t, int>, std::vector<std::pair<int64_t, int>>, std::greater<std::pair<int64_t, int>>> load;
    for (int b = 0; b < blocks; ++b) load.push({0, b});
    for (const auto& pc : by_cost) {
        const int i = pc.second, n_tiles = (int)((descs[i].N + 127) / 128);
        for (int j = 0; j < n_tiles; ++j) {
            auto top = load.top();
            load.pop();
            lists[(size_t)top.second].push_back(tile0[i] + j);
            top.first += -pc.first;
            load.push(top);
        }
    }
    int pos = 0;
    for (int b = 0; b < blocks; ++b) {
        wg_start[b] = pos;
        for (int v : lists[(size_t)b]) tile_list[pos++] = v;
    }
    wg_start[blocks] = pos;
    if (hipMemcpyAsync(table, blob.data(), blob.size(), hipMemcpyHostToDevice, st) != hipSuccess) return BL_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return BL_ERR_HIP;   /* the host copy of the table dies here */
    memset(plan, 0, sizeof(*plan));
    plan->count = count;
    plan->blocks = blocks;
    plan->layout = layout;
    plan->wg_offset = (int64_t)L.wg_off;
    plan->prep_offset = (int64_t)L.list_off;
    plan->packed_bytes = packed_bytes;
    plan->table_bytes = (int64_t)bl_stack_table_bytes_batched(descs, count, M);
    plan->tokens = M;
    plan->entries = count;
    plan->red_ints = (int32_t)tiles;                      /* tiles of the whole table */
    plan->norm = 3;                                       /* the tile route */
    return BL_OK;
}

static std::atomic<bool> g_mb_attr_set;

static bl_status stack_build_batched(const bl_decode_desc* descs, int count, int layout, int M, void* table,
                                     bl_stack_plan* plan, hipStream_t st) {
    for (int i = 0; i < count; ++i) {
        const bl_status rc = check_batched_desc(descs[i], layout);
        if (rc != BL_OK) return rc;
    }
    int64_t entries64 = 0;
    size_t ws_bytes = 0;
    if (!mb_sizes(descs, count, M, &entries64, &ws_bytes)) return BL_ERR_SHAPE;
    if (mb_tile_route(descs, count, M)) return stack_build_tiles(descs, count, layout, M, table, plan, st);
    const int entries = (int)entries64;
    const mb_layout_t L = mb_layout(entries, count, ws_bytes);
    uint8_t* const dev_base = (uint8_t*)table;
    std::vector<bl_stream_item> items;
    std::vector<bl_mb_fin_item> fins;                    /* one per product that is split along k */
    std::vector<int> units_v;
    std::vector<int64_t> ucost_v, ecost_v;
    int64_t packed_bytes = 0, total_units = 0, max_elems = 0;
    int lds = 0, split_products = 0;
    size_t ws_used = 0;
    for (int i = 0; i < count; ++i) {
        const bl_decode_desc& d = descs[i];
        const int64_t Kp = bl_kpad(d.K);
        mb_split sp;
        mb_split_product(M, Kp, &sp);
        packed_bytes += d.N * (Kp / 4);
        int32_t* ws = nullptr;
        if (sp.parts > 1) {
            ws = (int32_t*)(dev_base + L.ws_off + ws_used);
            ws_used += align_up((size_t)((int64_t)M * d.N * 4), 256);
            ++split_products;
            if ((int64_t)M * d.N > max_elems) max_elems = (int64_t)M * d.N;
        }
        if (ws) fins.push_back(bl_mb_fin_item{ws, d.rowsum, d.scale, d.beta, d.residual, d.acc, d.y, M, (int)d.N});
        for (int g = 0; g < sp.groups; ++g) {
            const int m0 = g * sp.per_group, m = M - m0 < sp.per_group ? M - m0 : sp.per_group;
            for (int pt = 0; pt < sp.parts; ++pt) {
                const int c0 = pt * sp.part_chunks;
                const int nch = (int)(Kp / 64) - c0 < sp.part_chunks ? (int)(Kp / 64) - c0 : sp.part_chunks;
                bl_stream_item it;
                memset(&it, 0, sizeof(it));
                it.packed = (const bl_v4i*)d.packed;
                it.beta = d.beta;
                it.q = d.q + (int64_t)m0 * Kp;
                it.scale = d.scale ? d.scale + m0 : nullptr;
                it.rowsum = d.rowsum + m0;
                it.residual = d.residual ? d.residual + (int64_t)m0 * d.N : nullptr;
                it.acc = d.acc ? d.acc + (int64_t)m0 * d.N : nullptr;
                it.y = d.y ? d.y + (int64_t)m0 * d.N : nullptr;
                it.acc_ws = ws ? ws + (int64_t)m0 * d.N : nullptr;
                it.N = (int)d.N;
                it.nchunks = nch;
                it.row_chunks = (int)(Kp / 64);
                it.c0 = c0;
                it.ldq = (int)Kp;
                it.qgroups = (int)(Kp / 16);
                it.layout = layout;
                it.m = m;
                it.units = (int)((d.N + 31) / 32);
                const int need = (int)(m * (nch * 64 + 16) + BL_MB_MISC + BL_MB_WAVES * BL_MB_TILE);
                if (need > lds) lds = need;
                items.push_back(it);
                units_v.push_back(it.units);
                ucost_v.push_back((int64_t)32 * nch * 16);
                ecost_v.push_back((int64_t)2 * m * nch * 64);   /* staging the token rows */
                total_units += it.units;
            }
        }
    }
    lds = (lds + 255) / 256 * 256;
    bool two_tiles = false;
    for (int i = 0; i < count; ++i) {
        mb_split sp;
        mb_split_product(M, bl_kpad(descs[i].K), &sp);
        two_tiles = two_tiles || sp.per_group > 32;
    }
    const void* kern = two_tiles ? (const void*)bl_stream_mb<2> : (const void*)bl_stream_mb<1>;
    if (!g_mb_attr_set.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute((const void*)bl_stream_mb<1>, hipFuncAttributeMaxDynamicSharedMemorySize, BL_MB_LDS_MAX) !=
                hipSuccess ||
            hipFuncSetAttribute((const void*)bl_stream_mb<2>, hipFuncAttributeMaxDynamicSharedMemorySize, BL_MB_LDS_MAX) !=
                hipSuccess)
            return BL_ERR_HIP;
        g_mb_attr_set.store(true, std::memory_order_release);
    }
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, BL_MB_THREADS, (size_t)lds) !=
            hipSuccess ||
        cus < 1 || per_cu < 1)
        return BL_ERR_HIP;
    int64_t blocks64 = (int64_t)cus * per_cu;
    if (blocks64 > (total_units + BL_MB_WAVES - 1) / BL_MB_WAVES) blocks64 = (total_units + BL_MB_WAVES - 1) / BL_MB_WAVES;
    if (blocks64 > BL_STREAM_MAX_BLOCKS) blocks64 = BL_STREAM_MAX_BLOCKS;
    if (blocks64 < 1) blocks64 = 1;
    const int blocks = (int)blocks64;
    const std::vector<int2> wg = cut_slices(units_v, ucost_v, ecost_v, blocks);
    std::vector<uint8_t> blob(L.ws_off, 0);
    memcpy(blob.data(), items.data(), items.size() * sizeof(bl_stream_item));
    memcpy(blob.data() + L.wg_off, wg.data(), wg.size() * sizeof(int2));
    if (!fins.empty()) memcpy(blob.data() + L.fin_off, fins.data(), fins.size() * sizeof(bl_mb_fin_item));
    /* the partial sums start at zero; every run leaves them at zero again */
    if (ws_bytes && hipMemsetAsync(dev_base + L.ws_off, 0, ws_bytes, st) != hipSuccess) return BL_ERR_HIP;
    if (hipMemcpyAsync(table, blob.data(), blob.size(), hipMemcpyHostToDevice, st) != hipSuccess) return BL_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return BL_ERR_HIP;   /* the host copy of the table dies here */
    memset(plan, 0, sizeof(*plan));
    plan->count = count;
    plan->blocks = blocks;
    plan->lds_bytes = lds;
    plan->layout = layout;
    plan->wg_offset = (int64_t)L.wg_off;
    plan->prep_offset = (int64_t)L.fin_off;
    plan->packed_bytes = packed_bytes;
    plan->table_bytes = (int64_t)L.total;
    plan->tokens = M;
    plan->entries = entries;
    plan->prep_count = split_products;                  /* > 0: the finishing kernel runs */
    plan->red_ints = (int32_t)((max_elems + 1023) / 1024);   /* its grid in x */
    plan->norm = two_tiles ? 2 : 1;                       /* token tiles of the kernel variant */
    return BL_OK;
}

extern "C" size_t bl_stack_table_bytes(const bl_decode_desc* descs, int count) {
    if (!descs || count < 1 || count > BL_STACK_MAX_COUNT) return 0;
    size_t q_bytes = 0, acc_bytes = 0;
    for (int i = 0; i < count; ++i) {
        if (descs[i].K < 1 || descs[i].K > 64 * 64 * BL_STREAM_LMAX || descs[i].N < 1 || descs[i].N > (1 << 28)) return 0;
        if (desc_is_fused(descs[i])) q_bytes += align_up((size_t)descs[i].K, 256);
        acc_bytes += align_up((size_t)descs[i].N * 4, 256);     /* partial sums of the k-major form */
    }
    return stream_layout(count, q_bytes, acc_bytes).total;
}

extern "C" bl_status bl_stack_build(const bl_decode_desc* descs, int count, int layout, int64_t M, void* table,
                                    bl_stack_plan* plan, bl_stream s) {
    if (!descs || !table || !plan) return BL_ERR_NULL;
    if (count < 1 || count > BL_STACK_MAX_COUNT || M < 1 || M > BL_STACK_MAX_TOKENS) return BL_ERR_SHAPE;
    if (!bl_aligned(table, 256)) return BL_ERR_ALIGN;
    if (M > 1) return stack_build_batched(descs, count, layout, (int)M, table, plan, (hipStream_t)s);
    size_t q_bytes = 0, acc_bytes = 0;
    for (int i = 0; i < count; ++i) {
        const bl_status st = check_stack_desc(descs[i], layout);
        if (st != BL_OK) return st;
        if (desc_is_fused(descs[i])) q_bytes += align_up((size_t)descs[i].K, 256);
        acc_bytes += align_up((size_t)descs[i].N * 4, 256);
    }
    const bl_stream_layout L = stream_layout(count, q_bytes, acc_bytes);
    uint8_t* const dev_base = (uint8_t*)table;
    std::vector<bl_stream_item> items((size_t)count);
    std::vector<bl_stream_prep_item> preps;
    int inline_count = 0, max_chunks = 0, max_units = 0, max_cols = 0;
    size_t acc_used = 0;
    std::vector<int64_t> unit_bytes((size_t)count);
    bool any_norm = false;
    int64_t total = 0, packed_bytes = 0, total_units = 0;
    size_t q_used = 0;
    for (int i = 0; i < count; ++i) {
        const bl_decode_desc& d = descs[i];
        const bool fused = desc_is_fused(d);
        const int64_t Kp = bl_kpad(d.K);                 /* row length of the packed weights and of q */
        bl_stream_item it;
        memset(&it, 0, sizeof(it));
        it.packed = (const bl_v4i*)d.packed;
        it.beta = d.beta;
        it.residual = d.residual;
        it.acc = d.acc;
        it.y = d.y;
        it.N = (int)d.N;
        /* 16-byte loads per weight row: 64 weights each, or 80 in the five-per-byte form */
        const int64_t row_bytes = layout == BL_LAYOUT_TRIT5    ? bl_kpad5(d.K) / 5
                                  : layout == BL_LAYOUT_KMAJOR ? (d.N + 63) / 64 * 16
                                                               : Kp / 4;
        it.nchunks = (int)(row_bytes / 16);
        it.qgroups = (int)(Kp / 16);
        if (it.nchunks > max_chunks) max_chunks = it.nchunks;
        it.layout = layout;
        int lgG = 3;
        while (((it.nchunks + (1 << lgG) - 1) >> lgG) > BL_STREAM_LMAX) ++lgG;   /* K bound checked: lgG <= 6 */
        int R = 64 >> lgG;
        it.lgG = lgG;
        it.lp = (it.nchunks + (1 << lgG) - 1) >> lgG;
        it.units = (it.N + R - 1) / R;
        if (layout == BL_LAYOUT_KMAJOR) {
            /* one row per k: dword columns of 16 output features; a unit is 64 consecutive k */
            const int ncols = (int)((d.N + 63) / 64 * 4);
            it.nchunks = ncols;
            it.lp = (ncols + 63) / 64;
            it.units = (int)(Kp / 64);
            it.acc_ws = (int32_t*)(dev_base + L.acc_off + acc_used);
            acc_used += align_up((size_t)d.N * 4, 256);
            if (it.units > max_units) max_units = it.units;
            if (ncols > max_cols) max_cols = ncols;
            R = 64;                                          /* weight rows of a unit */
        }
        if (fused && d.prod.in0 == nullptr) {
            /* a plain bf16 row: quantised inside the stream launch by each workgroup that meets it */
            it.xbf16 = d.X;
            it.q_out = d.q_out;
            it.scale_out = d.scale_out;
            it.fixed_scale = d.fixed_scale;
            it.rowsum_pub = (int32_t*)(dev_base + L.rowsum_off) + i;
            it.scale_pub = (float*)(dev_base + L.scale_off) + i;
            if (layout == BL_LAYOUT_KMAJOR) {                /* read back by the finishing kernel */
                it.rowsum = it.rowsum_pub;
                it.scale = it.scale_pub;
            }
            ++inline_count;
        } else if (fused || !d.rowsum) {
            bl_stream_prep_item pp;
            memset(&pp, 0, sizeof(pp));
            pp.K = (int)Kp;
            pp.rowsum_ws = (int32_t*)(dev_base + L.rowsum_off) + i;
            it.rowsum = pp.rowsum_ws;
            if (fused) {
                pp.fused = 1;
                if (!bl_make_prod(d.prod, d.X, d.K, &pp.prod)) return BL_ERR_VALUE;
                any_norm = any_norm || pp.prod.norm;
                pp.q_ws = (int8_t*)(dev_base + L.q_off + q_used);
                q_used += align_up((size_t)d.K, 256);
                pp.scale_ws = (float*)(dev_base + L.scale_off) + i;
                pp.q_out = d.q_out;
                pp.scale_out = d.scale_out;
                pp.fixed_scale = d.fixed_scale;
                it.q = pp.q_ws;
                it.scale = pp.scale_ws;
            } else {
                pp.q_in = d.q;
                it.q = d.q;
                it.scale = d.scale;
            }
            preps.push_back(pp);
        } else {
            it.q = d.q;
            it.scale = d.scale;
            it.rowsum = d.rowsum;
        }
        it.rowsum_fin = it.rowsum;
        it.scale_fin = it.scale ? it.scale : it.beta;        /* unused without y; a valid address */
        unit_bytes[(size_t)i] = (int64_t)R * row_bytes;
        total += (int64_t)it.units * unit_bytes[(size_t)i];
        total_units += it.units;
        packed_bytes += (layout == BL_LAYOUT_KMAJOR ? d.K : d.N) * row_bytes;
        items[(size_t)i] = it;
    }
    /* persistent grid: the workgroups that are resident at once, but no more than one per four
     * row groups' worth of work (a workgroup has four waves) */
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &per_cu,
            layout == BL_LAYOUT_TRIT5    ? (const void*)bl_stream_m1_t5
            : layout == BL_LAYOUT_KMAJOR ? (const void*)bl_stream_m1_km
                                         : (const void*)bl_stream_m1,
            256,
            (size_t)BL_STREAM_LDS_BYTES) != hipSuccess ||
        cus < 1 || per_cu < 1)
        return BL_ERR_HIP;
    int64_t blocks64 = (int64_t)cus * per_cu;
    if (blocks64 > (total_units + 3) / 4) blocks64 = (total_units + 3) / 4;
    if (blocks64 > BL_STREAM_MAX_BLOCKS) blocks64 = BL_STREAM_MAX_BLOCKS;
    if (blocks64 < 1) blocks64 = 1;
    const int blocks = (int)blocks64;

    /* Slice boundaries: a workgroup's time is its bytes, weighted by the measured rate of the
     * product's register shape, plus a fixed cost each time it enters a product (activation
     * row, pipeline refill; larger when it quantises the row itself), expressed in bytes at a
     * workgroup's share of the stream rate. */
    std::vector<int> units_v((size_t)count);
    std::vector<int64_t> ucost_v((size_t)count), ecost_v((size_t)count);
    for (int i = 0; i < count; ++i) {
        units_v[(size_t)i] = items[(size_t)i].units;
        ucost_v[(size_t)i] = items[(size_t)i].lp == 5 ? unit_bytes[(size_t)i] : unit_bytes[(size_t)i] * 26 / 25;
        ecost_v[(size_t)i] = items[(size_t)i].xbf16 ? (int64_t)36 << 10 : (int64_t)12 << 10;
    }
    const std::vector<int2> wg = cut_slices(units_v, ucost_v, ecost_v, blocks);
    std::vector<uint8_t> blob(L.rowsum_off, 0);
    memcpy(blob.data(), items.data(), items.size() * sizeof(bl_stream_item));
    memcpy(blob.data() + L.wg_off, wg.data(), wg.size() * sizeof(int2));
    if (!preps.empty()) memcpy(blob.data() + L.prep_off, preps.data(), preps.size() * sizeof(bl_stream_prep_item));
    hipStream_t st = (hipStream_t)s;
    /* the k-major form's partial sums start at zero; every run leaves them at zero again */
    if (layout == BL_LAYOUT_KMAJOR && hipMemsetAsync(dev_base + L.acc_off, 0, acc_bytes, st) != hipSuccess)
        return BL_ERR_HIP;
    if (hipMemcpyAsync(table, blob.data(), blob.size(), hipMemcpyHostToDevice, st) != hipSuccess) return BL_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return BL_ERR_HIP;   /* the host copy of the table dies here */

    memset(plan, 0, sizeof(*plan));
    plan->count = count;
    plan->blocks = blocks;
    plan->prep_count = (int32_t)preps.size();
    plan->inline_count = inline_count;
    plan->norm = any_norm ? 1 : 0;
    plan->lds_bytes = BL_STREAM_LDS_BYTES;
    plan->layout = layout;
    plan->red_ints = layout == BL_LAYOUT_KMAJOR ? max_cols * 16 : 0;
    plan->wg_offset = (int64_t)L.wg_off;
    plan->prep_offset = (int64_t)L.prep_off;
    plan->packed_bytes = packed_bytes;
    plan->table_bytes = (int64_t)L.total;
    plan->tokens = 1;
    plan->entries = count;
    return BL_OK;
}

extern "C" bl_status bl_stack_run(void* table, const bl_stack_plan* plan, bl_stream s) {
    if (!table || !plan) return BL_ERR_NULL;
    if (plan->tokens > 1 && plan->norm == 3) {               /* the tile route of the batched form */
        if (plan->tokens < BL_MB_TILE_ROUTE_MIN || plan->tokens > BL_STACK_MAX_TOKENS || plan->count < 1 ||
            plan->count > BL_STACK_MAX_COUNT || plan->entries != plan->count || plan->red_ints < plan->count ||
            plan->blocks < 1 || plan->blocks > plan->red_ints || plan->blocks > BL_STREAM_MAX_BLOCKS ||
            plan->layout != BL_LAYOUT_K16 || plan->prep_count != 0)
            return BL_ERR_VALUE;
        const tile_layout_t Lt = tile_layout(plan->count, plan->red_ints);
        if (plan->wg_offset != (int64_t)Lt.wg_off || plan->prep_offset != (int64_t)Lt.list_off) return BL_ERR_VALUE;
        if (!bl_aligned(table, 256)) return BL_ERR_ALIGN;
        const uint8_t* tb = (const uint8_t*)table;
        return bl_gemm_table_launch((const bl_tile_item*)tb, (const int*)(tb + Lt.t0_off), plan->count, plan->red_ints,
                                    plan->tokens, plan->blocks, (const int*)(tb + Lt.wg_off),
                                    (const int*)(tb + Lt.list_off), s);
    }
    if (plan->tokens > 1) {
        if (plan->tokens > BL_STACK_MAX_TOKENS || plan->count < 1 || plan->count > BL_STACK_MAX_COUNT ||
            plan->entries < plan->count || plan->entries > 64 * BL_STACK_MAX_COUNT || plan->blocks < 1 ||
            plan->blocks > BL_STREAM_MAX_BLOCKS || plan->lds_bytes < BL_MB_MISC + BL_MB_WAVES * BL_MB_TILE || plan->lds_bytes > BL_MB_LDS_MAX ||
            plan->lds_bytes % 256 || plan->layout != BL_LAYOUT_K16)
            return BL_ERR_VALUE;
        const mb_layout_t Lb = mb_layout(plan->entries, plan->count, 0);
        if (plan->wg_offset != (int64_t)Lb.wg_off || plan->prep_offset != (int64_t)Lb.fin_off || plan->prep_count < 0 ||
            plan->prep_count > plan->count || plan->red_ints < 0 || (plan->prep_count > 0 && plan->red_ints < 1) ||
            plan->norm < 1 || plan->norm > 2)
            return BL_ERR_VALUE;
        if (!bl_aligned(table, 256)) return BL_ERR_ALIGN;
        if (!g_mb_attr_set.load(std::memory_order_acquire)) return BL_ERR_VALUE;   /* no table was built in this process */
        const uint8_t* tb = (const uint8_t*)table;
        if (plan->norm == 2)
            bl_stream_mb<2><<<plan->blocks, BL_MB_THREADS, (size_t)plan->lds_bytes, (hipStream_t)s>>>(
                (const bl_stream_item*)tb, (const int2*)(tb + Lb.wg_off));
        else
            bl_stream_mb<1><<<plan->blocks, BL_MB_THREADS, (size_t)plan->lds_bytes, (hipStream_t)s>>>(
                (const bl_stream_item*)tb, (const int2*)(tb + Lb.wg_off));
        if (hipGetLastError() != hipSuccess) return BL_ERR_HIP;
        if (plan->prep_count > 0)
            bl_mb_finish<<<dim3((unsigned)plan->red_ints, (unsigned)plan->prep_count), 256, 0, (hipStream_t)s>>>(
                (const bl_mb_fin_item*)(tb + Lb.fin_off));
        return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
    }
    if (plan->count < 1 || plan->count > BL_STACK_MAX_COUNT || plan->blocks < 1 ||
        plan->blocks > BL_STREAM_MAX_BLOCKS || plan->prep_count < 0 || plan->inline_count < 0 ||
        plan->prep_count + plan->inline_count > plan->count || plan->lds_bytes < 64 ||
        plan->lds_bytes > 48 * 1024 || plan->lds_bytes % 16 ||
        plan->layout < 0 || plan->layout > BL_LAYOUT_KMAJOR || plan->red_ints < 0 || plan->red_ints > BL_KM_MAX_N ||
        (plan->layout == BL_LAYOUT_KMAJOR && (plan->red_ints < 64 || plan->lds_bytes < 64 + 64 + plan->red_ints * 4)))
        return BL_ERR_VALUE;
    const bl_stream_layout L = stream_layout(plan->count, 0);
    if (plan->wg_offset != (int64_t)L.wg_off || plan->prep_offset != (int64_t)L.prep_off) return BL_ERR_VALUE;
    if (!bl_aligned(table, 256)) return BL_ERR_ALIGN;
    uint8_t* base = (uint8_t*)table;
    hipStream_t st = (hipStream_t)s;
    if (plan->prep_count > 0) {
        const bl_stream_prep_item* pp = (const bl_stream_prep_item*)(base + L.prep_off);
        if (plan->norm) bl_stream_prep<true><<<plan->prep_count, 256, 0, st>>>(pp);
        else bl_stream_prep<false><<<plan->prep_count, 256, 0, st>>>(pp);
        if (hipGetLastError() != hipSuccess) return BL_ERR_HIP;
    }
    if (plan->layout == BL_LAYOUT_KMAJOR) {
        bl_stream_m1_km<<<plan->blocks, 256, (size_t)plan->lds_bytes, st>>>(
            (const bl_stream_item*)base, (const int2*)(base + L.wg_off), (plan->lds_bytes - 64) / 4 - plan->red_ints,
            plan->red_ints);
        if (hipGetLastError() != hipSuccess) return BL_ERR_HIP;
        bl_km_finish<<<dim3((unsigned)((plan->red_ints + 255) / 256), (unsigned)plan->count), 256, 0, st>>>(
            (const bl_stream_item*)base);
    } else if (plan->layout == BL_LAYOUT_TRIT5)
        bl_stream_m1_t5<<<plan->blocks, 256, (size_t)plan->lds_bytes, st>>>(
            (const bl_stream_item*)base, (const int2*)(base + L.wg_off), (plan->lds_bytes - 64) / 4);
    else
        bl_stream_m1<<<plan->blocks, 256, (size_t)plan->lds_bytes, st>>>(
            (const bl_stream_item*)base, (const int2*)(base + L.wg_off), (plan->lds_bytes - 64) / 4);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}
