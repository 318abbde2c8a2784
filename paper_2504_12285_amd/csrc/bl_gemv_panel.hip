/* Batched-decode W1.58A8 product for 3..64 tokens with int8 inputs (Section 5.1 of
 * the BitNet b1.58 2B4T report: packed weights streamed from HBM once, unpacked on chip
 * right before the int8 product).
 *
 * With this many tokens a workgroup can no longer keep every token row in LDS.  The kernel is
 * a skinny GEMM: eight waves walk the k axis in steps of KS = 512 (256 is kept for comparisons:
 * 13.1 / 15.3 us per layer at M = 32 / 64 against 10.5 / 13.9; half the barriers, waits and
 * address arithmetic per k); both operands travel global -> LDS by direct loads (no registers)
 * through a ring of S stages, S-1 of them in flight.
 *
 * What bounds it is LDS time, and that shaped the work split.  Measured on this kernel's loop
 * skeleton: a CU takes direct-load data into LDS at ~48 B/clk and serves ds_read_b128 at ~138
 * B/clk, and the two do NOT overlap (24 KB of direct loads + 80 KB of reads per step cost
 * 506 + 570 clk).  So every staged byte should be read from LDS once: a wave owns one token
 * block (32 tokens) and one k part of each step and multiplies it against ALL row blocks of
 * the workgroup (NI = 1, 2 or 4 blocks of 32 rows, v_mfma_i32_32x32x32_i8, NI accumulators);
 * the eight waves are TB token blocks (1: M <= 32, 2: M <= 64) x KH = 8/TB k parts, and the k
 * parts meet through LDS once at the end, where all eight waves share the sums and the stores.
 *
 * LDS stage: TB*32 token rows of KS bytes, then 32*NI weight rows of KS/4 packed bytes.
 * 16-byte units are XOR-swizzled against the row index (applied to the global address a lane
 * fetches, since a direct load writes 64 consecutive units), which spreads the reads of both
 * operands over the banks.  Inside a k step lane half h and MFMA s use packed word (KS/32)*h+s
 * (16 consecutive k); k part kh takes NSUB = KS/32/KH consecutive s.
 *
 * Offset codes: the matrix cores multiply codes 0..2; sum_k q (given, or accumulated by one
 * more chain against an all-ones operand) is subtracted once per output. */
#include <atomic>

#include <type_traits>

#include "bl_device.h"
#include "bl_gemv_common.h"
#include "bl_host.h"

#define BL_PANEL_HEAD 128   /* ints in front of the ring: 64 token scales, 64 row sums */

typedef int bl_v2i __attribute__((ext_vector_type(2)));

template <int TB, int S, bool NEED_SUM, int NI, int KS>
__device__ __forceinline__ void bl_panel_body(const bl_gemv_prob& P, const int M, int* lds) {
    static_assert(KS == 256 || KS == 512, "k step");
    constexpr int UA = KS / 16;                            /* 16-byte units of a token row per step */
    constexpr int UW = KS / 64;                            /* 16-byte units of a packed row per step */
    constexpr int RPP = 1024 / KS;                         /* token rows per 1 KB piece */
    constexpr int SA = TB * 32 * KS, SW = 128 * (KS / 4), STG = SA + SW;
    constexpr int NA = TB * (KS / 256);                    /* activation loads per wave and stage */
    constexpr int NWL = (NI * UW * 4 + 63) / 64;           /* weight loads per wave and stage */
    constexpr int LOADS = NA + NWL;                        /* direct loads per wave and stage */
    constexpr int KH = 8 / TB, NSUB = (KS / 32) / KH;      /* k parts; MFMA sub-steps per wave and step */
    static_assert((S - 2) * LOADS < 64, "vmcnt is a 6-bit count");
    static_assert(S * STG >= 8 * 4 * 4096, "the ring must hold the partial sums of the epilogue");
    const int N = P.N, K = P.K;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int tb = w % TB, kh = w / TB;
    const int n_base = ((int)blockIdx.x - P.block0) * (NI * 32);
    const int wunits = K / 64;                             /* 16-byte units per packed row */
    const int nsteps = (K + KS - 1) / KS;
    float* fscale = (float*)lds;
    int* frs = lds + 64;
    uint8_t* ring = (uint8_t*)(lds + BL_PANEL_HEAD);

    /* The token scales and row sums go to LDS by direct loads too (wave 0, one dword per lane,
     * ahead of every stage load: loads return in order, so they have landed when the first
     * stage has).  No register waits for them. */
    const float bt = *P.beta;
    if (w == 0) {
        const int t = lane < M ? lane : M - 1;
        if (P.scale) __builtin_amdgcn_global_load_lds((bl_gptr)(P.scale + t), (bl_lptr)fscale, 4, 0, 0);
        if (!NEED_SUM) __builtin_amdgcn_global_load_lds((bl_gptr)(P.rowsum + t), (bl_lptr)frs, 4, 0, 0);
    }

    /* Per-lane sources of the direct loads, computed once: a k step only adds its offset.
     * Exactly LOADS instructions per wave and stage whatever the shape, so that the vmcnt
     * immediates below are right: tokens beyond M re-read row M-1, rows beyond N re-read row
     * N-1 (never stored), and in a last, partial k step the units beyond K re-read the step's
     * first unit (their weights are zeroed at the point of use). */
    constexpr int WPW = NI * UW * 4;                       /* weight units per wave and stage */
    const int nl = WPW < 64 ? WPW : 64;                    /* lanes of a weight load in use */
    const int8_t* asrc[NA];
    int au[NA];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int row = (w * NA + j) * RPP + lane / UA;    /* piece w*NA+j: RPP token rows = 1 KB */
        const int tok = row < M ? row : M - 1;
        au[j] = (lane % UA) ^ (row & 15);
        asrc[j] = P.q + (int64_t)tok * K + au[j] * 16;
    }
    const bl_v4i* wsrc[NWL];
    int wunit[NWL];
#pragma unroll
    for (int jj = 0; jj < NWL; ++jj) {
        const int U = w * WPW + jj * 64 + lane;            /* unit of the stage's weight region */
        const int row = U / UW;
        wunit[jj] = (U % UW) ^ (UW == 4 ? (row >> 2) & 3 : (row >> 1) & 7);
        int n = n_base + row;
        if (n >= N) n = N - 1;
        wsrc[jj] = P.packed + (int64_t)n * wunits + wunit[jj];
    }
    auto issue = [&](int ks, int buf) {
        uint8_t* base = ring + buf * STG;
        /* wave-uniform: only the last step can be partial, and only then are sources clamped (the
         * full steps pay one 64-bit add per load and nothing else) */
        if (ks * KS + KS > K) {
#pragma unroll
            for (int j = 0; j < NA; ++j) {
                const int8_t* src = asrc[j] + ks * KS;
                if (ks * KS + au[j] * 16 >= K) src -= au[j] * 16;
                __builtin_amdgcn_global_load_lds((bl_gptr)src, (bl_lptr)(base + (w * NA + j) * 1024), 16, 0, 0);
            }
            if (lane < nl) {
#pragma unroll
                for (int jj = 0; jj < NWL; ++jj) {
                    const bl_v4i* src = wsrc[jj] + ks * UW;
                    if (ks * UW + wunit[jj] >= wunits) src -= wunit[jj];
                    __builtin_amdgcn_global_load_lds((bl_gptr)src, (bl_lptr)(base + SA + (w * WPW + jj * 64) * 16), 16,
                                                     0, 0);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < NA; ++j)
                __builtin_amdgcn_global_load_lds((bl_gptr)(asrc[j] + ks * KS), (bl_lptr)(base + (w * NA + j) * 1024), 16,
                                                 0, 0);
            if (lane < nl) {
#pragma unroll
                for (int jj = 0; jj < NWL; ++jj)
                    __builtin_amdgcn_global_load_lds((bl_gptr)(wsrc[jj] + ks * UW),
                                                     (bl_lptr)(base + SA + (w * WPW + jj * 64) * 16), 16, 0, 0);
            }
        }
    };

    bl_v16i C[NI], Cs;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) C[ni][v] = 0;
#pragma unroll
    for (int v = 0; v < 16; ++v) Cs[v] = 0;

    /* per-lane LDS read offsets inside a stage: this wave's MFMA sub-steps are s = kh*TB + j,
     * packed word / activation unit 8h + s */
    const int u0 = h * (KS / 32) + kh * NSUB;              /* first word (and activation unit) of the wave */
    const int ar = tb * 32 + l32;                          /* token row in the stage */
    int a_off[NSUB];
#pragma unroll
    for (int j = 0; j < NSUB; ++j) a_off[j] = ar * KS + (((u0 + j) ^ (ar & 15)) * 16);
    /* weight row l32 of block ni sits at (ni*32 + l32) * KS/4; its unit u0/4 is swizzled with
     * row bits that do not depend on ni */
    const int w_off = SA + l32 * (KS / 4) +
                      (((u0 >> 2) ^ (UW == 4 ? (l32 >> 2) & 3 : (l32 >> 1) & 7)) * 16) + (u0 & 3) * 4;

    auto compute = [&](int ks, int buf, auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;   /* a partial last step: mask the words beyond K */
        const uint8_t* st = ring + buf * STG;
        bl_v4i a[NSUB];
#pragma unroll
        for (int j = 0; j < NSUB; ++j) a[j] = *(const bl_v4i*)(st + a_off[j]);
        uint32_t wds[NI][NSUB];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            {
                if constexpr (NSUB == 4) {
                    const bl_v4i q4 = *(const bl_v4i*)(st + w_off + ni * 32 * (KS / 4));
#pragma unroll
                    for (int j = 0; j < 4; ++j) wds[ni][j] = (uint32_t)q4[j];
                } else if constexpr (NSUB == 2) {
                    const bl_v2i q2 = *(const bl_v2i*)(st + w_off + ni * 32 * (KS / 4));
                    wds[ni][0] = (uint32_t)q2[0];
                    wds[ni][1] = (uint32_t)q2[1];
                } else {
                    wds[ni][0] = (uint32_t)*(const int*)(st + w_off + ni * 32 * (KS / 4));
                }
            }
        }
        const int k0 = ks * KS;
#pragma unroll
        for (int j = 0; j < NSUB; ++j) {
            const bool cv = !TAIL || k0 + (u0 + j) * 16 < K;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                {
                    const uint32_t wd = cv ? wds[ni][j] : 0u;
                    uint32_t l0 = wd & 0x03030303u, l1 = (wd >> 2) & 0x03030303u, l2 = (wd >> 4) & 0x03030303u,
                             l3 = (wd >> 6) & 0x03030303u;
                    if (P.layout == 0) bl_transpose4x4(l0, l1, l2, l3);
                    const bl_v4i b = {(int)l0, (int)l1, (int)l2, (int)l3};
                    C[ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[j], b, C[ni], 0, 0, 0);
                }
            }
            if (NEED_SUM) {
                const int one = cv ? 0x01010101 : 0;
                const bl_v4i ones = {one, one, one, one};
                Cs = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[j], ones, Cs, 0, 0, 0);
            }
        }
    };

    for (int s0 = 0; s0 < S - 1 && s0 < nsteps; ++s0) issue(s0, s0);
    for (int it = 0; it < nsteps; ++it) {
        /* stage `it` has landed; the stages issued after it may stay in flight */
        const int later = nsteps - 1 - it;
        bl_wait_stages<S - 2, LOADS>(later < S - 2 ? later : S - 2);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        const int nx = it + S - 1;
        if (nx < nsteps) issue(nx, nx % S);
        if (it * KS + KS > K) compute(it, it % S, std::true_type());
        else compute(it, it % S, std::false_type());
    }

    bl_mfma_fence();
    asm volatile("" ::: "memory");
    __syncthreads();                                       /* every wave is done with the ring */
    /* The k parts meet in LDS: wave w leaves its partial sums (minus its part of sum_k q) for
     * each row block, then wave wv = nib*TB + tbb adds the KH parts of block (tbb, nib),
     * rescales and stores: all eight waves share the epilogue when NI*TB = 8. */
    bl_v4i* red = (bl_v4i*)ring;                           /* [wave][ni][4][64] groups of four sums */
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        {
            bl_v16i Dp = C[ni];
            if (NEED_SUM) Dp -= Cs;
#pragma unroll
            for (int vq = 0; vq < 4; ++vq)
                red[((w * NI + ni) * 4 + vq) * 64 + lane] = bl_v4i{Dp[4 * vq], Dp[4 * vq + 1], Dp[4 * vq + 2], Dp[4 * vq + 3]};
        }
    }
    __syncthreads();
    const int tbb = w % TB, nib = w / TB;
    const int n = n_base + nib * 32 + l32;
    if (nib < NI && n < N) {
        bl_v16i D;
#pragma unroll
        for (int v = 0; v < 16; ++v) D[v] = 0;
#pragma unroll
        for (int kp = 0; kp < KH; ++kp)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const bl_v4i t4 = red[(((kp * TB + tbb) * NI + nib) * 4 + vq) * 64 + lane];
#pragma unroll
                for (int e = 0; e < 4; ++e) D[4 * vq + e] += t4[e];
            }
        /* The token terms come from LDS four at a time; residual values first, then the stores
         * back to back (a load between two stores would make each store wait for the one before
         * it: stores count on vmcnt too), through global-address-space pointers, y and acc in
         * loops of their own so that the wave-uniform tests stay outside. */
        typedef __attribute__((address_space(1))) float* gfloat_p;
        typedef __attribute__((address_space(1))) int* gint_p;
        typedef const __attribute__((address_space(1))) float* gcfloat_p;
        auto emit = [&](auto add_tag) {
            constexpr bool ADD = decltype(add_tag)::value;
            int val[16];
            float cf[16];
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int t0 = tbb * 32 + vq * 8 + h * 4;
                const float4 sc4 = *(const float4*)(fscale + t0);
                const float scv[4] = {sc4.x, sc4.y, sc4.z, sc4.w};
                bl_v4i rs4 = {0, 0, 0, 0};
                if (!NEED_SUM) rs4 = *(const bl_v4i*)(frs + t0);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    val[4 * vq + e] = D[4 * vq + e] - rs4[e];
                    cf[4 * vq + e] = bt * scv[e];
                }
            }
            if (P.y) {
                gfloat_p yp = (gfloat_p)P.y + n;
                float res[16];
                if (ADD) {
                    gcfloat_p rp = (gcfloat_p)P.residual + n;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int tok = tbb * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
                        res[v] = rp[(int64_t)(tok < M ? tok : M - 1) * N];
                    }
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int tok = tbb * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
                    const float r = (float)val[v] * cf[v];
                    if (tok < M) yp[(int64_t)tok * N] = ADD ? res[v] + r : r;
                }
            }
            if (P.acc) {
                gint_p ap = (gint_p)P.acc + n;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int tok = tbb * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
                    if (tok < M) ap[(int64_t)tok * N] = val[v];
                }
            }
        };
        if (P.y && P.residual) emit(std::true_type());
        else emit(std::false_type());
    }
}

/* NI is a property of the workgroup's product: one specialised body per value, so that the
 * accumulators are a fixed set of registers. */
template <int TB, int S, bool NEED_SUM, int KS>
__global__ __launch_bounds__(512) void bl_gemv_panel(const bl_gemv_group grp, const int M) {
    extern __shared__ __attribute__((aligned(16))) int lds[];
    const bl_gemv_prob P = bl_fetch_prob(grp);
    if (P.ksplit == 4) bl_panel_body<TB, S, NEED_SUM, 4, KS>(P, M, lds);
    else if (P.ksplit == 2) bl_panel_body<TB, S, NEED_SUM, 2, KS>(P, M, lds);
    else bl_panel_body<TB, S, NEED_SUM, 1, KS>(P, M, lds);
}

template <int TB, int S, int KS>
static bl_status launch_panel(const bl_gemv_group& grp, int M, int blocks, bool have_sums, hipStream_t st) {
    constexpr int lds = BL_PANEL_HEAD * 4 + S * (TB * 32 * KS + 128 * (KS / 4));
    static_assert(lds <= 160 * 1024, "LDS of one CU");
    auto kern = have_sums ? bl_gemv_panel<TB, S, false, KS> : bl_gemv_panel<TB, S, true, KS>;
    /* (two threads may both set the attribute: the call is idempotent) */
    static std::atomic<bool> done[2];
    if (!done[have_sums].load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return BL_ERR_HIP;
        done[have_sums].store(true, std::memory_order_release);
    }
    kern<<<blocks, 512, lds, st>>>(grp, M);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

/* M <= 64, int8 inputs only.  Rows per workgroup: 32 * NI.  A long k gets NI = 1: its
 * workgroups stream the most activation bytes and would otherwise finish last (measured on
 * the four shapes of a layer at M = 64: 18.9 us against 22.4 with NI = 2); every NI is halved
 * while the launch would leave most CUs without a workgroup. */
bl_status bl_gemv_panel_launch(bl_gemv_group& grp, int M, hipStream_t st) {
    if (M < 1 || M > 64) return BL_ERR_SHAPE;
    const int TB = M <= 32 ? 1 : 2;
    bool have_sums = true;
    int blocks = 0;
    for (int div = 1; div <= 4; div *= 2) {
        blocks = 0;
        bool floor_all = true;
        for (int i = 0; i < grp.count; ++i) {
            bl_gemv_prob& P = grp.p[i];
            if (P.fused || !P.q) return BL_ERR_SHAPE;
            if (!P.rowsum) have_sums = false;
            int ni = (P.K > 4096 ? 1 : 4) / div;
            if (ni <= 1) ni = 1;
            else floor_all = false;
            P.ksplit = ni;
            P.block0 = blocks;
            blocks += (P.N + 32 * ni - 1) / (32 * ni);
        }
        if (blocks >= 128 || floor_all) break;
    }
    return TB == 1 ? launch_panel<1, 4, 512>(grp, M, blocks, have_sums, st)
                   : launch_panel<2, 3, 512>(grp, M, blocks, have_sums, st);
}
