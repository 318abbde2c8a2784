/* Internal device helpers shared by the HIP kernels of the BitLinear library
 * (not part of the public boundary).  gfx950 only: 64-lane wavefronts. */
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bitlinear.h"

typedef int bl_v4i __attribute__((ext_vector_type(4)));
typedef int bl_v16i __attribute__((ext_vector_type(16)));

#define BL_WAVE 64

/* bf16 bit pattern -> fp32 (exact). */
__device__ __forceinline__ float bl_bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

/* fp32 -> bf16 bit pattern, round to nearest even (finite inputs). */
__device__ __forceinline__ uint32_t bl_f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

/* Correctly rounded fp32 quotient: the fp64 quotient of two fp32 values,
 * rounded to fp32, equals the directly rounded fp32 quotient (53 >= 2*24+2). */
__device__ __forceinline__ float bl_div_rn(float a, float b) { return (float)((double)a / (double)b); }

/* DPP cross-lane moves inside a row of 16 lanes (old value = 0 for disabled lanes). */
template <int CTRL>
__device__ __forceinline__ int bl_dpp(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
#define BL_DPP_QUAD_XOR1 0xB1   /* quad_perm [1,0,3,2] */
#define BL_DPP_QUAD_XOR2 0x4E   /* quad_perm [2,3,0,1] */
#define BL_DPP_ROW_HALF_MIRROR 0x141
#define BL_DPP_ROW_MIRROR 0x140

/* Sum over aligned groups of G lanes (G = 4, 8 or 16), result in every lane of
 * the group.  DPP only: quad butterflies, then half-row / row mirrors (after a
 * quad sum all four lanes of a quad agree, so a mirror pairs distinct quads). */
template <int G>
__device__ __forceinline__ int bl_group_sum(int v) {
    static_assert(G == 1 || G == 2 || G == 4 || G == 8 || G == 16, "group size");
    if (G >= 2) v += bl_dpp<BL_DPP_QUAD_XOR1>(v);
    if (G >= 4) v += bl_dpp<BL_DPP_QUAD_XOR2>(v);
    if (G >= 8) v += bl_dpp<BL_DPP_ROW_HALF_MIRROR>(v);
    if (G >= 16) v += bl_dpp<BL_DPP_ROW_MIRROR>(v);
    return v;
}

/* Full-wave integer sum / float max via butterflies (ds_bpermute for the
 * cross-row steps). */
__device__ __forceinline__ int bl_wave_sum(int v) {
    v = bl_group_sum<16>(v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}
__device__ __forceinline__ float bl_wave_max(float v) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

/* 4x4 byte transpose of four dwords: out[s].byte[b] = in[b].byte[s]. */
__device__ __forceinline__ void bl_transpose4x4(uint32_t& a0, uint32_t& a1, uint32_t& a2, uint32_t& a3) {
    const uint32_t t0 = __builtin_amdgcn_perm(a1, a0, 0x05010400u);
    const uint32_t t1 = __builtin_amdgcn_perm(a1, a0, 0x07030602u);
    const uint32_t t2 = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
    a0 = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    a1 = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    a2 = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    a3 = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

/* Direct global->LDS loads (16 bytes per lane): the LDS destination is a wave-uniform
 * base, lane l's bytes land at base + 16*l.  They count on vmcnt like any load. */
typedef const __attribute__((address_space(1))) void* bl_gptr;
typedef __attribute__((address_space(3))) void* bl_lptr;

/* s_waitcnt vmcnt(n) only, n < 64: expcnt = 7, lgkmcnt = 15 left open (gfx9 encoding:
 * vmcnt bits 3:0 in imm[3:0], bits 5:4 in imm[15:14]) */
#define BL_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
/* s_waitcnt lgkmcnt(0) only (vmcnt = 63 and expcnt = 7 left open): a wave's own LDS writes have
 * been performed.  A raw s_barrier does not imply it, so a wave that hands data to other waves
 * through LDS waits with this in front of the barrier. */
#define BL_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt(0xC07F)

/* Waits until at most r stages of LOADS direct loads each are still in flight (r <= J). */
template <int J, int LOADS>
__device__ __forceinline__ void bl_wait_stages(int r) {
    if (r >= J) {
        BL_WAIT_VM(J * LOADS);
    } else {
        if constexpr (J > 0) bl_wait_stages<J - 1, LOADS>(r);
    }
}

/* Expand one packed word (16 weights, layout-1 digit order) into the sixteen
 * int8 codes of 16 consecutive k: three shifts and four masks. */
__device__ __forceinline__ bl_v4i bl_unpack16(uint32_t p) {
    bl_v4i b;
    b[0] = (int)(p & 0x03030303u);
    b[1] = (int)((p >> 2) & 0x03030303u);
    b[2] = (int)((p >> 4) & 0x03030303u);
    b[3] = (int)((p >> 6) & 0x03030303u);
    return b;
}

/* Wait for in-flight matrix-core results before ordinary vector instructions
 * read an accumulator.  The hardware has no interlock for that read, and the
 * compiler's wait-state count for the gfx950 16x16x64 int8 MFMA proved too
 * short on hardware (the last result rows were read before they were written).
 * 32 idle issue cycles cover the longest (16-pass) MFMA; the scheduling
 * barriers keep every MFMA before and every reader after this point. */
__device__ __forceinline__ void bl_mfma_fence() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}
