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
#include <atomic>

#include "bl_device.h"
#include "bl_gemv_common.h"
#include "bl_host.h"
#include "bl_producer.h"

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
template <int M, int G, int L, bool NORM>
__global__ __launch_bounds__(256) void bl_gemv_rows(const bl_gemv_group grp) {
    extern __shared__ int lds[];
    constexpr int R = 64 / G;
    const bl_gemv_prob P = bl_fetch_prob(grp);
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
    const bool pre_bf16 = P.fused && P.prod.kind == BL_PROD_BF16 && !(NORM && P.prod.norm);
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
    /* small loads go out before the weight stream and are used late */
    const float bt = *P.beta;
    float sc_in = 0.0f;
    int rs_in = 0;
    if (!P.fused && tid < M) {
        if (P.scale) sc_in = P.scale[tid];
        if (P.rowsum) rs_in = P.rowsum[tid];
    }

    bl_v4i p[L];
    const bl_v4i* wrow = P.packed + (int64_t)(row_ok ? n : 0) * nchunks;
#pragma unroll
    for (int i = 0; i < L; ++i) {
        const int chunk = (i * ksplit + kp) * G + g;
        p[i] = bl_v4i{0, 0, 0, 0};
        if (row_ok && chunk < nchunks) p[i] = __builtin_nontemporal_load(wrow + chunk);
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
            float rn = 1.0f;
            bool have_xv = pre_bf16 && m == 0;
            if (NORM && P.prod.norm) {
                rn = bl_norm_produce2(P.prod, m, K, first_block, (double*)red, xv);
                have_xv = true;
            }
            float mx = 0.0f;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = tid + j * 256;
                if (u < groups) {
                    if (!have_xv) bl_produce16<NORM>(P.prod, m, u, K, first_block, rn, xv[2 * j], xv[2 * j + 1]);
                    mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(xv[2 * j]), bl_absmax8_bf16(xv[2 * j + 1])));
                }
            }
            for (int u = tid + 512; u < groups; u += 256) {
                uint4 lo, hi;
                bl_produce16<NORM>(P.prod, m, u, K, false, rn, lo, hi);
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
                bl_produce16<NORM>(P.prod, m, u, K, first_block, rn, lo, hi);
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
            sq[tid] = rs_in;
            fs[tid] = sc_in;
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

#define BL_MMA_PAD 16    /* bytes added to each staged activation row (LDS bank spread) */
#define BL_MMA_HEAD 144  /* ints in front of the rows: 4 wave maxima, 64 token scales, 64 row sums */

/* Matrix-core decode kernel, M <= 16*MT tokens, up to four products per launch.
 * Same work split as bl_gemv_rows with G = 4: lane (c, kg) owns weight row c of
 * a 16-row group and k chunks (i*ksplit+kp)*4+kg, and issues all of its 16-byte
 * weight loads first.  Each packed word d of a chunk is opened into its four
 * bit-pair levels by shift and mask (plus a 4x4 byte transpose for layout 0),
 * which puts the sixteen codes of k = 16d .. 16d+15 in natural order: the B
 * operand of one v_mfma_i32_16x16x64_i8 whose A operand is sixteen consecutive
 * int8 of token l%16, read from LDS rows that hold q as it is in memory.  The k
 * reduction happens inside the matrix core: no cross-lane step.  sum_k q comes
 * from a second chain with an all-ones B operand when no rowsum was given.
 * Tokens beyond M read the last real row (their results are never stored).
 *
 * int8 inputs: the rows are staged 1024 << LF columns at a time (so that 64
 * tokens fit), wave w copying tokens/column blocks w, w+4, ..; the loads of the
 * next phase are in flight during the products of the current one.  Fused
 * inputs: produced, quantised and staged whole, one token at a time.
 * Dynamic LDS: BL_MMA_HEAD ints, then max(M*(row+16), MT*4096) bytes. */
template <int L, int MT, bool NEED_SUM, bool NORM>
__global__ __launch_bounds__(256) void bl_gemv_mma(const bl_gemv_group grp, const int M, const int LF, const int budget) {
    extern __shared__ int lds[];
    const bl_gemv_prob P = bl_fetch_prob(grp);
    const int N = P.N, K = P.K, nchunks = K / 64, ksplit = P.ksplit;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, kg = lane >> 4;
    const int rg = w / ksplit, kp = w - rg * ksplit;
    const int rows_per_block = (4 / ksplit) * 16;
    const int n = ((int)blockIdx.x - P.block0) * rows_per_block + rg * 16 + c;
    const bool row_ok = n < N;
    const int groups = K / 16;
    const bool fused = P.fused != 0;
    /* int8 inputs: everything at once when M rows of K fit the LDS budget, else two
     * buffers of PK = 1024 << LF columns (the launcher sized LF so that a phase is 64
     * (token, 1024-column) pieces: 16 loads per wave) */
    const bool whole = fused || M * (K + BL_MMA_PAD) <= budget;
    const int PK = whole ? K : (1024 << LF);              /* columns per staging phase */
    const int qstride = PK + BL_MMA_PAD;                  /* bytes per staged token row */
    const int bufsz = M * qstride;
    float* fs = (float*)lds;                              /* 4 wave maxima              */
    float* fscale = fs + 4;                               /* M <= 64 input scales       */
    int* frs = (int*)(fscale + 64);                       /* M <= 64 input row sums     */
    uint8_t* Q = (uint8_t*)(lds + BL_MMA_HEAD);
    int* red = (int*)Q;                                   /* D of 4 waves, MT tiles: reuses the rows */

    /* Workgroups run in step and all want the same rows: each starts at a different phase
     * and a different piece, so that at any moment they ask different L2 channels. */
    const int nph = (K + PK - 1) / PK;
    const int rot_ph = (int)blockIdx.x % nph;
    constexpr int NS = 16;                                /* loads per wave and phase (phased mode) */
    /* phase php of the phased mode into buffer buf: exactly NS loads per wave, so that the
     * vmcnt immediates below are right; a piece outside M x kw re-loads piece (0, 0) */
    auto stage_phase = [&](int php, int buf) {
        const int k0 = php * PK, kw = K - k0 < PK ? K - k0 : PK;
        uint8_t* base = Q + buf * bufsz;
        const int rot_j = ((int)blockIdx.x / nph) & (NS - 1);
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const int t = w + 4 * ((j + rot_j) & (NS - 1));
            int m = t >> LF, jj = t & ((1 << LF) - 1);
            if (m >= M || jj * 1024 >= kw) m = jj = 0;
            const int c16 = lane + 64 * jj;
            if (c16 * 16 < kw)
                __builtin_amdgcn_global_load_lds((bl_gptr)(P.q + (int64_t)m * K + k0 + c16 * 16),
                                                 (bl_lptr)(base + m * qstride + jj * 1024), 16, 0, 0);
        }
    };
    /* whole mode: wave w copies pieces w, w+4, .. of the M x ceil(K/1024) grid, rotated */
    auto stage_whole = [&]() {
        const int cols = (K + 1023) / 1024, pieces = M * cols;
        const int rot = (int)(blockIdx.x * 5u) % pieces;
        for (int t = w; t < pieces; t += 4) {
            const int tt = t + rot < pieces ? t + rot : t + rot - pieces;
            const int m = tt / cols, jj = tt - m * cols;
            const int c16 = lane + 64 * jj;
            if (c16 * 16 < K)
                __builtin_amdgcn_global_load_lds((bl_gptr)(P.q + (int64_t)m * K + c16 * 16),
                                                 (bl_lptr)(Q + m * qstride + jj * 1024), 16, 0, 0);
        }
    };

    /* 1. activation loads first (token 0 of the fused path, or the first phase of q) */
    uint4 xv[4];
    const bool pre_bf16 = fused && P.prod.kind == BL_PROD_BF16 && !(NORM && P.prod.norm);
    const bool first_block = blockIdx.x == (unsigned)P.block0;
    /* without normalisation every wave quantises tokens w, w+4, .. on its own: lane l holds
     * groups l and l+64 of the wave's first token */
    if (pre_bf16 && w < M) {
        const uint4* xr = (const uint4*)((const uint16_t*)P.prod.in0 + (int64_t)w * K);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int u = lane + j * 64;
            if (u < groups) {
                xv[2 * j] = xr[2 * u];
                xv[2 * j + 1] = xr[2 * u + 1];
            }
        }
    }
    /* small loads go out now and are used late: nothing below waits for them alone */
    const float bt = *P.beta;
    float sc_in = 0.0f;
    int rs_in = 0;
    if (!fused && tid < M) {
        if (P.scale) sc_in = P.scale[tid];
        if (P.rowsum) rs_in = P.rowsum[tid];
    }

    /* 2. every weight load of this wave.  The matrix core wants lane 16*kg+c to hold chunk kg
     * of row c, but four consecutive lanes should fetch 64 consecutive bytes: lane l loads
     * chunk l%4 of row l/4, and a lane permutation at the point of use puts it in place. */
    bl_v4i p[L];
    {
        const int lrow = lane >> 2, lkg = lane & 3;
        const int ln = n - c + lrow;                      /* the row this lane fetches */
        const bool lok = ln < N;
        const bl_v4i* wrow = P.packed + (int64_t)(lok ? ln : 0) * nchunks;
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int chunk = (i * ksplit + kp) * 4 + lkg;
            p[i] = bl_v4i{0, 0, 0, 0};
            if (lok && chunk < nchunks) p[i] = __builtin_nontemporal_load(wrow + chunk);
        }
    }
    const int perm_src = (4 * c + kg) * 4;                /* byte index of the lane that fetched for this one */

    if (!fused) {
        if (whole) {
            stage_whole();
        } else {
            stage_phase(rot_ph, 0);
            stage_phase(rot_ph + 1 < nph ? rot_ph + 1 : 0, 1);   /* nph >= 2 in phased mode */
        }
    }
    /* 3. fused path: produce, quantise and stage every token.  Without normalisation a token
     * is one wave's work (absmax by a wave reduction, no workgroup barrier per token): the four
     * waves run four tokens side by side.  A lane keeps its first two groups in registers
     * between the absmax pass and the quantising pass and produces the others twice. */
    if (fused && !(NORM && P.prod.norm)) {
#pragma unroll 1
        for (int m = w; m < M; m += 4) {
            const bool have_xv = pre_bf16 && m == w;
            float mx = 0.0f;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = lane + j * 64;
                if (u < groups) {
                    if (!have_xv) bl_produce16<NORM>(P.prod, m, u, K, first_block, 1.0f, xv[2 * j], xv[2 * j + 1]);
                    mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(xv[2 * j]), bl_absmax8_bf16(xv[2 * j + 1])));
                }
            }
            if (pre_bf16) {
                /* plain bf16 rows: the lane's other groups four at a time, so that their loads
                 * are in flight together (one round trip instead of four) */
                const uint4* xr = (const uint4*)((const uint16_t*)P.prod.in0 + (int64_t)m * K);
                for (int u0 = lane + 128; u0 < groups; u0 += 256) {
                    uint4 t[8];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (u0 + 64 * j < groups) {
                            t[2 * j] = xr[2 * (u0 + 64 * j)];
                            t[2 * j + 1] = xr[2 * (u0 + 64 * j) + 1];
                        }
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (u0 + 64 * j < groups)
                            mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(t[2 * j]), bl_absmax8_bf16(t[2 * j + 1])));
                }
            } else {
                for (int u = lane + 128; u < groups; u += 64) {
                    uint4 lo, hi;
                    bl_produce16<NORM>(P.prod, m, u, K, false, 1.0f, lo, hi);
                    mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(lo), bl_absmax8_bf16(hi)));
                }
            }
            const float gamma = bl_wave_max(mx);
            const float gg = fmaxf(gamma, 1e-5f);
            const float inv = bl_div_rn(127.0f, gg);
            const bool emit = P.q_out && first_block;
            uint8_t* Qm = Q + m * qstride;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = lane + j * 64;
                if (u < groups) {
                    uint32_t a0, a1, a2, a3;
                    bl_quant8_words(xv[2 * j], inv, a0, a1);
                    bl_quant8_words(xv[2 * j + 1], inv, a2, a3);
                    if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                    *(uint4*)(Qm + u * 16) = make_uint4(a0, a1, a2, a3);
                }
            }
            if (pre_bf16) {
                const uint4* xr = (const uint4*)((const uint16_t*)P.prod.in0 + (int64_t)m * K);
                for (int u0 = lane + 128; u0 < groups; u0 += 256) {
                    uint4 t[8];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (u0 + 64 * j < groups) {
                            t[2 * j] = xr[2 * (u0 + 64 * j)];
                            t[2 * j + 1] = xr[2 * (u0 + 64 * j) + 1];
                        }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int u = u0 + 64 * j;
                        if (u < groups) {
                            uint32_t a0, a1, a2, a3;
                            bl_quant8_words(t[2 * j], inv, a0, a1);
                            bl_quant8_words(t[2 * j + 1], inv, a2, a3);
                            if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                            *(uint4*)(Qm + u * 16) = make_uint4(a0, a1, a2, a3);
                        }
                    }
                }
            } else {
                for (int u = lane + 128; u < groups; u += 64) {
                    uint32_t a0, a1, a2, a3;
                    uint4 lo, hi;
                    bl_produce16<NORM>(P.prod, m, u, K, first_block, 1.0f, lo, hi);
                    bl_quant8_words(lo, inv, a0, a1);
                    bl_quant8_words(hi, inv, a2, a3);
                    if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                    *(uint4*)(Qm + u * 16) = make_uint4(a0, a1, a2, a3);
                }
            }
            if (lane == 0) {
                const float sc = bl_div_rn(gg, 127.0f);
                fscale[m] = P.fixed_scale > 0.0f ? P.fixed_scale : sc;
                if (P.scale_out && first_block) P.scale_out[m] = sc;
            }
        }
        __syncthreads();
    } else if (fused) {
#pragma unroll 1
        for (int m = 0; m < M; ++m) {
            float rn = 1.0f;
            bool have_xv = false;
            if (NORM && P.prod.norm) {
                rn = bl_norm_produce2(P.prod, m, K, first_block, (double*)frs, xv);
                have_xv = true;
            }
            float mx = 0.0f;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = tid + j * 256;
                if (u < groups) {
                    if (!have_xv) bl_produce16<NORM>(P.prod, m, u, K, first_block, rn, xv[2 * j], xv[2 * j + 1]);
                    mx = fmaxf(mx, fmaxf(bl_absmax8_bf16(xv[2 * j]), bl_absmax8_bf16(xv[2 * j + 1])));
                }
            }
            for (int u = tid + 512; u < groups; u += 256) {
                uint4 lo, hi;
                bl_produce16<NORM>(P.prod, m, u, K, false, rn, lo, hi);
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
            uint8_t* Qm = Q + m * qstride;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = tid + j * 256;
                if (u < groups) {
                    uint32_t a0, a1, a2, a3;
                    bl_quant8_words(xv[2 * j], inv, a0, a1);
                    bl_quant8_words(xv[2 * j + 1], inv, a2, a3);
                    if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                    *(uint4*)(Qm + u * 16) = make_uint4(a0, a1, a2, a3);
                }
            }
            for (int u = tid + 512; u < groups; u += 256) {
                uint32_t a0, a1, a2, a3;
                uint4 lo, hi;
                bl_produce16<NORM>(P.prod, m, u, K, first_block, rn, lo, hi);
                bl_quant8_words(lo, inv, a0, a1);
                bl_quant8_words(hi, inv, a2, a3);
                if (emit) *(uint4*)(P.q_out + (int64_t)m * K + u * 16) = make_uint4(a0, a1, a2, a3);
                *(uint4*)(Qm + u * 16) = make_uint4(a0, a1, a2, a3);
            }
            if (tid == 0) {
                const float sc = bl_div_rn(gg, 127.0f);
                fscale[m] = P.fixed_scale > 0.0f ? P.fixed_scale : sc;
                if (P.scale_out && first_block) P.scale_out[m] = sc;
            }
        }
        __syncthreads();
    }

    /* 4. products */
    constexpr bool need_sum = NEED_SUM;   /* the launcher checked: no product of the group has a rowsum */
    /* one accumulator per packed word d: four independent MFMA chains per token tile */
    bl_v4i C[MT][4], Cs[MT][2];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        C[t][0] = C[t][1] = C[t][2] = C[t][3] = bl_v4i{0, 0, 0, 0};
        Cs[t][0] = Cs[t][1] = bl_v4i{0, 0, 0, 0};
    }
    int arow[MT];                                         /* byte offset of this lane's token row */
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int tok = t * 16 + c;
        arow[t] = (tok < M ? tok : M - 1) * qstride;
    }
    /* one load step: chunk (i*ksplit+kp)*4+kg of this lane's row against the staged rows at
     * qb, whose column 0 is k0.  A lane whose chunk lies beyond K has zero weights and reads
     * column 0. */
    auto step = [&](const bl_v4i praw, int i, const uint8_t* qb, int k0, bool fence) {
        bl_v4i pw;
#pragma unroll
        for (int d = 0; d < 4; ++d) pw[d] = __builtin_amdgcn_ds_bpermute(perm_src, praw[d]);
        const int chunk = (i * ksplit + kp) * 4 + kg;
        const bool cv = chunk < nchunks;
        const int coff = cv ? chunk * 64 - k0 : 0;
        bl_v4i a[MT][4];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int d = 0; d < 4; ++d) a[t][d] = *(const bl_v4i*)(qb + arow[t] + coff + d * 16);
        const int one = cv ? 0x01010101 : 0;
        const bl_v4i ones = {one, one, one, one};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t wd = (uint32_t)pw[d];
            if (fence) asm volatile("" : "+v"(wd));       /* unpack here, not hoisted out of the phase loop */
            uint32_t l0 = wd & 0x03030303u, l1 = (wd >> 2) & 0x03030303u, l2 = (wd >> 4) & 0x03030303u,
                     l3 = (wd >> 6) & 0x03030303u;
            if (P.layout == 0) bl_transpose4x4(l0, l1, l2, l3);
            const bl_v4i b = {(int)l0, (int)l1, (int)l2, (int)l3};
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                C[t][d] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[t][d], b, C[t][d], 0, 0, 0);
                if (need_sum)
                    Cs[t][d & 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[t][d], ones, Cs[t][d & 1], 0, 0, 0);
            }
        }
    };
    if (nph == 1) {
        /* everything is staged at once: the first half of the load steps is in range for every
         * wave (L is the smallest variant that covers K), so that part is straight-line code */
        if (!fused) {
            BL_WAIT_VM(0);
            asm volatile("" ::: "memory");
            if (tid < M) {
                fscale[tid] = sc_in;
                frs[tid] = rs_in;
            }
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < L; ++i)
            if (i < L / 2 || (i * ksplit + kp) * 256 < K) step(p[i], i, Q, 0, false);
    } else {
        for (int ph = 0; ph < nph; ++ph) {
            const int php = ph + rot_ph < nph ? ph + rot_ph : ph + rot_ph - nph;
            const int k0 = php * PK;                      /* first k of this phase */
            const uint8_t* qb = Q + (ph & 1) * bufsz;
            /* this phase has landed (the next one, issued after it, may still be in flight) */
            if (ph + 1 < nph) BL_WAIT_VM(NS);
            else BL_WAIT_VM(0);
            asm volatile("" ::: "memory");
            if (ph == 0 && tid < M) {
                fscale[tid] = sc_in;
                frs[tid] = rs_in;
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < L; ++i) {
                const int kfirst = (i * ksplit + kp) * 256;   /* wave-uniform: first k of this step */
                if (kfirst >= k0 && kfirst < k0 + PK && kfirst < K) step(p[i], i, qb, k0, true);
            }
            if (ph + 2 < nph) {
                asm volatile("" ::: "memory");
                __syncthreads();                          /* every wave is done with this buffer */
                const int nx = ph + 2 + rot_ph;
                stage_phase(nx < nph ? nx : nx - nph, ph & 1);
            }
        }
    }
    bl_v4i D[MT];
    bl_mfma_fence();
#pragma unroll
    for (int t = 0; t < MT; ++t) D[t] = (C[t][0] + C[t][1]) + (C[t][2] + C[t][3]) - (Cs[t][0] + Cs[t][1]);

    if (ksplit > 1) {
        __syncthreads();                                  /* every wave is done reading the rows */
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
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const bl_v4i rs4 = *(const bl_v4i*)(frs + t * 16 + kg * 4);
            const float4 sc4 = *(const float4*)(fscale + t * 16 + kg * 4);
            const float scv[4] = {sc4.x, sc4.y, sc4.z, sc4.w};
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int tok = t * 16 + kg * 4 + v;
                if (tok < M) {
                    const int val = D[t][v] - (need_sum ? 0 : rs4[v]);
                    if (P.acc) P.acc[(int64_t)tok * N + n] = val;
                    if (P.y) {
                        const float r = (float)val * (bt * scv[v]);
                        P.y[(int64_t)tok * N + n] = P.residual ? P.residual[(int64_t)tok * N + n] + r : r;
                    }
                }
            }
        }
    }
}

template <int M, int G, int L, bool NORM>
static bl_status launch_rows(const bl_gemv_group& grp, int blocks, int maxK, hipStream_t st) {
    const size_t lds = (size_t)M * maxK + (size_t)M * 4 + (size_t)(M + 4) * 4 + (size_t)64 * M * 4;
    if (lds > 64 * 1024) return BL_ERR_SHAPE;
    bl_gemv_rows<M, G, L, NORM><<<blocks, 256, lds, st>>>(grp);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

template <int M, int G, bool NORM = false>
static bl_status launch_rows_l(int L, const bl_gemv_group& grp, int blocks, int maxK, hipStream_t st) {
    if (L <= 2) return launch_rows<M, G, 2, NORM>(grp, blocks, maxK, st);
    if (L <= 4) return launch_rows<M, G, 4, NORM>(grp, blocks, maxK, st);
    if (L <= 8) return launch_rows<M, G, 8, NORM>(grp, blocks, maxK, st);
    if (L <= 16) return launch_rows<M, G, 16, NORM>(grp, blocks, maxK, st);
    return launch_rows<M, G, 32, NORM>(grp, blocks, maxK, st);
}

template <int L, int MT, bool NORM = false>
static bl_status launch_mma(const bl_gemv_group& grp, int M, int blocks, hipStream_t st) {
    /* LDS budget for the staged rows: nearly all of it when every workgroup gets a CU of its
     * own, else small enough for two workgroups per CU.  int8 inputs that do not fit whole
     * are staged 1024 << LF columns at a time in two buffers; a phase is at most 64
     * (token, 1024-column) pieces: the kernel's 16 loads per wave. */
    const int budget = 150 * 1024;
    int LF = 0;
    while ((M << (LF + 1)) <= 64 && 2 * (size_t)M * ((1024 << (LF + 1)) + BL_MMA_PAD) <= (size_t)budget) ++LF;
    bool have_sums = true;   /* every product brings its own row sums */
    size_t rows = (size_t)MT * 4096;
    for (int i = 0; i < grp.count; ++i) {
        const bl_gemv_prob& P = grp.p[i];
        if (P.fused || !P.rowsum) have_sums = false;
        size_t need = (size_t)M * (P.K + BL_MMA_PAD);
        if (!P.fused && need > (size_t)budget) need = 2 * (size_t)M * ((1024 << LF) + BL_MMA_PAD);
        if (need > rows) rows = need;
    }
    const size_t lds = rows + BL_MMA_HEAD * 4;
    /* normalising producers are fused inputs: those never bring row sums */
    auto kern = NORM ? bl_gemv_mma<L, MT, true, NORM>
                     : (have_sums ? bl_gemv_mma<L, MT, false, false> : bl_gemv_mma<L, MT, true, false>);
    if (lds > 160 * 1024) return BL_ERR_SHAPE;
    if (lds > 64 * 1024) {
        /* (two threads may both set the attribute: the call is idempotent) */
        static std::atomic<bool> done[2];
        if (!done[have_sums].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) !=
                hipSuccess)
                return BL_ERR_HIP;
            done[have_sums].store(true, std::memory_order_release);
        }
    }
    kern<<<blocks, 256, lds, st>>>(grp, M, LF, budget);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

template <int MT, bool NORM = false>
static bl_status launch_mma_l(int L, const bl_gemv_group& grp, int M, int blocks, hipStream_t st) {
    if (L <= 2) return launch_mma<2, MT, NORM>(grp, M, blocks, st);
    if (L <= 4) return launch_mma<4, MT, NORM>(grp, M, blocks, st);
    if (L <= 8) return launch_mma<8, MT, NORM>(grp, M, blocks, st);
    if (L <= 16) return launch_mma<16, MT, NORM>(grp, M, blocks, st);
    return launch_mma<32, MT, NORM>(grp, M, blocks, st);
}

/* Lays the products of a group out over workgroups and launches them.  All
 * products of a group share M.  k is split over the waves of a workgroup when
 * a product alone would give fewer than about 150 workgroups.
 * Path: the VALU dot4 + DPP kernel for M <= 2, the matrix-core kernel above that (measured on
 * the four shapes of a layer in one launch, fused inputs: 7.4 / 14.0 / 18.6 / 23.0 us at M = 1..4
 * against 15.0 / 15.4 / 15.8 / 16.1; int8 inputs: 6.6 / 11.2 / 13.2 / 15.2 against 10.2 / 10.4 /
 * 10.6 / 10.8); normalising producers stay on the dot4 kernel up to M = 4.  The test hook
 * bl_debug_force_path forces one of them.  Returns BL_ERR_SHAPE if a K is too long for the register-resident row
 * scheme (the caller then uses the prefill kernel). */
bl_status bl_gemv_launch_group(bl_gemv_group& grp, int M, hipStream_t st) {
    const int forced = bl_forced_decode_path();   /* 0 default, 1 dot4, 2 row-resident, 3 panel */
    bool any_norm = false, any_fused = false;
    for (int i = 0; i < grp.count; ++i) {
        any_norm = any_norm || (grp.p[i].fused && grp.p[i].prod.norm);
        any_fused = any_fused || grp.p[i].fused;
    }
    /* (a group of int8 products at M = 2 already does better on the panel kernel: 9.9 against 11.2) */
    const bool dot4 = forced == 2   ? false
                      : forced == 1 ? M <= 4
                      : forced == 3 ? M <= 2 && any_fused
                                    : (M == 1 || (M == 2 && (any_fused || grp.count == 1)) || (M <= 4 && any_norm));
    const int G = dot4 ? 8 : 4;   /* lanes per weight row (8 measured better than 4 on the dot4 kernel) */
    /* workgroups wanted per product, measured: 150 for a product alone (best of 40..700) and
     * for the dot4 kernel; the matrix-core kernel, whose workgroups each stage all M rows,
     * does best with about 300 over the whole group */
    const int want_blocks = dot4 || grp.count < 2 ? 150 : 300 / grp.count;
    const int R = 64 / G;
    int blocks = 0, maxK = 0, L = 0;
    for (int i = 0; i < grp.count; ++i) {
        bl_gemv_prob& P = grp.p[i];
        int ks = 1;
        while (ks < 4 && (P.N + (4 / ks) * R - 1) / ((4 / ks) * R) < want_blocks) ks *= 2;
        P.ksplit = ks;
        P.block0 = blocks;
        const int rows_per_block = (4 / ks) * R;
        blocks += (P.N + rows_per_block - 1) / rows_per_block;
        if (P.K > maxK) maxK = P.K;
        const int l = (P.K / 64 + G * ks - 1) / (G * ks);
        if (l > L) L = l;
    }
    if (L > 32) return BL_ERR_SHAPE;
    if (any_norm) {
        /* normalising variants exist for the default lane split of the dot4 kernel and for
         * one token tile of the matrix-core kernel (fused inputs have M <= 16) */
        if (!dot4) return M <= 16 ? launch_mma_l<1, true>(L, grp, M, blocks, st) : BL_ERR_SHAPE;
        switch (M) {
            case 1: return launch_rows_l<1, 8, true>(L, grp, blocks, maxK, st);
            case 2: return launch_rows_l<2, 8, true>(L, grp, blocks, maxK, st);
            case 3: return launch_rows_l<3, 8, true>(L, grp, blocks, maxK, st);
            default: return launch_rows_l<4, 8, true>(L, grp, blocks, maxK, st);
        }
    }
    if (!dot4) {
        /* Matrix-core kernels.  The streaming panel kernel takes int8 inputs only; measured on
         * the four shapes of a layer (us per layer, row-resident kernel / panel kernel):
         *   one launch:  M = 3: 10.5 / 9.9, 8: 11.7 / 10.0, 16: 17.1 / 10.2, 32: 26.8 / 10.7, 48: 38.2 / 14.0
         *   four calls:  M = 8: 23.4 / 28.9, 16: 26.7 / 29.3, 24: 37.1 / 29.7, 48: 54.1 / 38.1
         * so a group goes to the panel kernel whenever it can, a product alone from 20 tokens. */
        const bool want_panel = !any_fused && (forced ? forced == 3 : (grp.count > 1 || M >= 20));
        if (want_panel) return bl_gemv_panel_launch(grp, M, st);
        if (M <= 16) return launch_mma_l<1>(L, grp, M, blocks, st);
        if (M <= 32) return launch_mma_l<2>(L, grp, M, blocks, st);
        return launch_mma_l<4>(L, grp, M, blocks, st);
    }
    switch (M) {
        case 1: return launch_rows_l<1, 8>(L, grp, blocks, maxK, st);
        case 2: return launch_rows_l<2, 8>(L, grp, blocks, maxK, st);
        case 3: return launch_rows_l<3, 8>(L, grp, blocks, maxK, st);
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
    K = bl_kpad(K);                 /* row length of the packed weights and of q */
    if (K > 8192)
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
    if (M < 1 || M > 64 || !bl_shape_ok(d.N, d.K) || d.K > 8192) return BL_ERR_SHAPE;
    if (fused && (M > 16 || d.K % 64 != 0 || M * (d.K + BL_MMA_PAD) > 96 * 1024)) return BL_ERR_SHAPE;
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
        P.N = (int)d.N; P.K = (int)bl_kpad(d.K); P.layout = layout; P.ksplit = 1; P.fixed_scale = d.fixed_scale;
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
