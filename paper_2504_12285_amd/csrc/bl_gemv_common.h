/* Internal: the product descriptor shared by the decode kernels (not part of the
 * public boundary). */
#pragma once
#include "bl_device.h"
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
    int ksplit;               /* waves sharing one row group (1, 2 or 4); in the    */
                              /* panel kernel: k parts of a k step (1, 2 or 4)      */
    float fixed_scale;        /* fused path: > 0 replaces absmax/127 in the rescale */
};
#define BL_GEMV_MAX_GROUP 4
struct bl_gemv_group {
    bl_gemv_prob p[BL_GEMV_MAX_GROUP];
    int count;
};

/* The descriptor of a workgroup's product, fetched from the kernel arguments ONCE and held in
 * scalar registers.  Without the pins the compiler re-reads a field from the argument
 * buffer at every use (a scalar-cache round trip in front of each store of the epilogue). */
template <typename T>
__device__ __forceinline__ void bl_pin(T& v) {
    asm volatile("" : "+s"(v));
}
__device__ __forceinline__ void bl_pin_prob(bl_gemv_prob& P) {
    bl_pin(P.packed); bl_pin(P.q); bl_pin(P.prod.kind); bl_pin(P.prod.in0); bl_pin(P.prod.in1);
    bl_pin(P.prod.aux_out); bl_pin(P.prod.voff); bl_pin(P.prod.group); bl_pin(P.prod.hd);
    bl_pin(P.prod.in_stride); bl_pin(P.fused); bl_pin(P.residual); bl_pin(P.beta); bl_pin(P.scale);
    bl_pin(P.rowsum); bl_pin(P.acc); bl_pin(P.y); bl_pin(P.q_out); bl_pin(P.scale_out); bl_pin(P.N);
    bl_pin(P.K); bl_pin(P.layout); bl_pin(P.block0); bl_pin(P.ksplit); bl_pin(P.fixed_scale);
}
__device__ __forceinline__ bl_gemv_prob bl_fetch_prob(const bl_gemv_group& grp) {
    int pi = 0;
#pragma unroll
    for (int i = 1; i < BL_GEMV_MAX_GROUP; ++i)
        if (i < grp.count && (int)blockIdx.x >= grp.p[i].block0) pi = i;
    bl_gemv_prob P = grp.p[pi];
    bl_pin_prob(P);
    return P;
}

/* Batched decode, 17..64 tokens with int8 inputs (bl_gemv_panel.hip): lays the products of
 * the group out over workgroups and launches them. */
bl_status bl_gemv_panel_launch(bl_gemv_group& grp, int M, hipStream_t st);
