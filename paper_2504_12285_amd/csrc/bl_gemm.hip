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

#include <atomic>

#define GEMM_THREADS 256

#define GEMM_PAD 16   /* bytes of padding per activation row in LDS (bank spread) */

/* Block tile BM x BN, k step BK (64 or 128), four waves arranged WGM x WGN.
 * LDS is double buffered: while the matrix cores work on buffer b, the next
 * k step travels global -> registers -> buffer 1-b; one barrier per k step.
 *   A buffer: BM rows x (BK + pad) int8 activations.
 *   W buffer: BN rows x (BK/16 + 1) packed words (16 weights each).
 * Operand mapping of v_mfma_i32_32x32x32_i8: lane l supplies 16 consecutive k
 * (offset 16*(l/32)) of row l%32 for both operands; a packed word expands to
 * exactly those 16 int8 (layout 1), so one ds_read_b32 feeds one B operand. */
template <int BM, int BN, int BK, int WGM, int LAYOUT>
__global__ __launch_bounds__(GEMM_THREADS) void bl_gemm_mfma(const uint8_t* __restrict__ packed,
                                                              const int8_t* __restrict__ q,
                                                              const int32_t* __restrict__ rowsum,
                                                              const float* __restrict__ beta,
                                                              const float* __restrict__ scale, int M, int N, int K,
                                                              const float* __restrict__ residual,
                                                              int32_t* __restrict__ acc, float* __restrict__ y) {
    constexpr int WGN = 4 / WGM;
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    constexpr int KS = BK / 32;                       /* MFMA k sub-steps per k step  */
    constexpr int A_STRIDE = BK + GEMM_PAD;           /* bytes                        */
    constexpr int W_WORDS = BK / 16;                  /* packed words per row, k step */
    constexpr int W_STRIDE = W_WORDS + 1;             /* dwords                       */
    constexpr int A_UPR = BK / 16;                    /* 16-byte units per A row      */
    constexpr int A_UNITS = BM * A_UPR / GEMM_THREADS;
    constexpr int W_UPR = BK / 64;                    /* 16-byte units per W row      */
    constexpr int W_UNITS = (BN * W_UPR + GEMM_THREADS - 1) / GEMM_THREADS;
    static_assert(BM * A_UPR % GEMM_THREADS == 0, "A tile must split evenly");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int A_BYTES = BM * A_STRIDE;
    constexpr int W_BYTES = BN * W_STRIDE * 4;
    auto As = [&](int b) { return smem + b * A_BYTES; };
    auto Ws = [&](int b) { return (uint32_t*)(smem + 2 * A_BYTES + b * W_BYTES); };

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int l32 = lane & 31, h = lane >> 5;
    const int kb = K / 4;

    bl_v16i C[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) C[mi][ni][v] = 0;

    uint4 areg[A_UNITS];
    uint4 wreg[W_UNITS];
    const uint8_t* aptr[A_UNITS];
    const uint8_t* wptr[W_UNITS];
#pragma unroll
    for (int i = 0; i < A_UNITS; ++i) {
        const int u = tid + i * GEMM_THREADS, row = u / A_UPR, c = u % A_UPR;
        int m = m0 + row;
        if (m >= M) m = M - 1;
        aptr[i] = (const uint8_t*)q + (int64_t)m * K + c * 16;
    }
#pragma unroll
    for (int i = 0; i < W_UNITS; ++i) {
        const int u = tid + i * GEMM_THREADS, row = u / W_UPR, c = u % W_UPR;
        int n = n0 + row;
        if (n >= N) n = N - 1;
        wptr[i] = packed + (int64_t)n * kb + c * 16;
    }

    auto load_tiles = [&](int kk) {
#pragma unroll
        for (int i = 0; i < A_UNITS; ++i) areg[i] = *(const uint4*)(aptr[i] + (int64_t)kk * BK);
#pragma unroll
        for (int i = 0; i < W_UNITS; ++i)
            if (tid + i * GEMM_THREADS < BN * W_UPR) wreg[i] = *(const uint4*)(wptr[i] + (int64_t)kk * (BK / 4));
    };
    auto store_tiles = [&](int b) {
#pragma unroll
        for (int i = 0; i < A_UNITS; ++i) {
            const int u = tid + i * GEMM_THREADS, row = u / A_UPR, c = u % A_UPR;
            uint32_t a0 = areg[i].x, a1 = areg[i].y, a2 = areg[i].z, a3 = areg[i].w;
            if (LAYOUT == 0) bl_transpose4x4(a0, a1, a2, a3);
            *(uint4*)(As(b) + row * A_STRIDE + c * 16) = make_uint4(a0, a1, a2, a3);
        }
#pragma unroll
        for (int i = 0; i < W_UNITS; ++i) {
            const int u = tid + i * GEMM_THREADS, row = u / W_UPR, c = u % W_UPR;
            if (u < BN * W_UPR) {
                uint32_t* d = Ws(b) + row * W_STRIDE + c * 4;
                d[0] = wreg[i].x; d[1] = wreg[i].y; d[2] = wreg[i].z; d[3] = wreg[i].w;
            }
        }
    };

    const int steps = K / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    for (int kk = 0; kk < steps; ++kk) {
        const int b = kk & 1;
        if (kk + 1 < steps) load_tiles(kk + 1);
        const uint8_t* Ab = As(b) + (wm0 + l32) * A_STRIDE + h * 16;
        const uint32_t* Wb = Ws(b) + (wn0 + l32) * W_STRIDE + h;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bl_v4i a[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) a[mi] = *(const bl_v4i*)(Ab + mi * 32 * A_STRIDE + ks * 32);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const uint32_t p = Wb[ni * 32 * W_STRIDE + ks * 2];
                bl_v4i bop;
                bop[0] = (int)(p & 0x03030303u);
                bop[1] = (int)((p >> 2) & 0x03030303u);
                bop[2] = (int)((p >> 4) & 0x03030303u);
                bop[3] = (int)((p >> 6) & 0x03030303u);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    C[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], bop, C[mi][ni], 0, 0, 0);
            }
        }
        if (kk + 1 < steps) store_tiles(b ^ 1);
        __syncthreads();
    }

    /* Epilogue: per-row terms through LDS once (see bl_gemm_tile256). */
    bl_mfma_fence();
    __syncthreads();
    int* rs_s = (int*)smem;
    float* cf_s = (float*)(smem + BM * 4);
    for (int i = tid; i < BM; i += GEMM_THREADS) {
        const int m = m0 + i;
        rs_s[i] = m < M ? rowsum[m] : 0;
        cf_s[i] = (y && m < M) ? *beta * scale[m] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int ml = wm0 + mi * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
            const int m = m0 + ml;
            if (m < M) {
                const int rs = rs_s[ml];
                const float c = cf_s[ml];
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const int n = n0 + wn0 + ni * 32 + l32;
                    if (n < N) {
                        const int val = C[mi][ni][v] - rs;
                        if (acc) acc[(int64_t)m * N + n] = val;
                        if (y) {
                            const float t = (float)val * c;
                            y[(int64_t)m * N + n] = residual ? residual[(int64_t)m * N + n] + t : t;
                        }
                    }
                }
            }
        }
}

template <int BM, int BN, int BK, int WGM>
static bl_status launch_gemm(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                             const float* scale, const int32_t* rowsum, int M, int N, int K,
                             const float* residual, int32_t* acc, float* y, hipStream_t st) {
    constexpr size_t lds = 2 * (size_t)(BM * (BK + GEMM_PAD) + BN * (BK / 16 + 1) * 4);
    dim3 grid((unsigned)((N + BN - 1) / BN), (unsigned)((M + BM - 1) / BM));
    auto k0 = bl_gemm_mfma<BM, BN, BK, WGM, 0>;
    auto k1 = bl_gemm_mfma<BM, BN, BK, WGM, 1>;
    auto kern = layout == 0 ? k0 : k1;
    if (lds > 64 * 1024) {
        /* (two threads may both set the attribute: the call is idempotent) */
        static std::atomic<bool> set[2];
        std::atomic<bool>& done = set[layout == 0 ? 0 : 1];
        if (!done.load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
                hipSuccess)
                return BL_ERR_HIP;
            done.store(true, std::memory_order_release);
        }
    }
    kern<<<grid, GEMM_THREADS, lds, st>>>(packed, q, rowsum, beta, scale, M, N, K, residual, acc, y);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

/* ---- large-tile pipelined kernel -------------------------------------------
 * 256 x 256 output tile per workgroup, k step 128, three LDS stages filled by
 * direct global->LDS loads (no register staging) two k steps ahead of the
 * matrix cores; one barrier per k step.  WM x WN waves (4 or 8 in total): with
 * eight waves every SIMD holds two, so one wave's unpack and LDS traffic hide
 * behind the other's MFMAs (a single wave reaches only ~60 % of the MFMA rate
 * once the unpack instructions share its issue slot).
 *
 * LDS stage = A part (BM rows x 128 int8, 16-byte units XOR-swizzled by
 * (row/2)%8) + W part (BN rows x 32 packed bytes = two units, swapped by row/8%2): with these
 * two patterns sixteen consecutive lanes of a ds_read_b128 fall on sixteen different 16-byte
 * bank groups (measured on a read-only loop, 8 waves per CU: 152 - 154 B/clk/CU against 113 - 116
 * for swizzles by row%8 and row/4%2, which are conflict-free only over eight lanes).
 * A direct load writes 64 consecutive units per wave, so the swizzle is applied
 * to the GLOBAL address each lane fetches, not to the LDS address.
 *
 * k mapping inside a k step: MFMA sub-step ks, lane half h  <->  the 16 k of
 * packed word 4h+ks (bytes 16*(4h+ks).. of the activation row).  Lane half h
 * therefore needs exactly unit h of a weight row: one ds_read_b128 per 32 rows
 * and k step, and one per (32 rows, sub-step) for the activations.
 *
 * Workgroups are numbered so that the 32 that share an XCD (and its L2) at a
 * time form an 8 x 4 patch of tiles: 8 activation row tiles x 4 weight tiles.
 * Requires layout 1, K % 128 == 0. */
#define G3_BK 128


/* EPI: 0 = plain epilogue (int32 and/or fp32 outputs, optional residual); 1 = fused producer
 * epilogue "residual": t = residual + product, written as fp32 (y, optional) and as bf16 (xb) with
 * the row maximum of |bf16(t)| folded into absmax[m]; 2 = "squared-ReLU gate": the tile's 128 weight
 * rows are 2 x 32 gate rows and the 2 x 32 matching up rows (n and N/2 + n), t = (relu(g)*relu(g))*u
 * for N/2 output columns, written as bf16 with its row maximum (Section 2: ReLU^2 in the FFN,
 * per-token absmax quantisation of the next BitLinear's input). */
/* TABLE: the persistent grid walks the tiles of a whole TABLE of products (device array `items`,
 * tile0[i] = first virtual tile of product i; at most BM token rows, so a tile is one block of
 * BN weight rows of one product) instead of the tiles of the one product in the arguments: the
 * batched decode of a stack of BitLinears in one launch whose weights are read once. */
/* DEFER: the fp32 outputs of a tile are not stored in a burst behind its k loop (every workgroup of
 * a launch reaches that point together, the chip then writes at the HBM rate while its matrix cores
 * idle: measured 19 - 23 thousand clocks of stores per 128 x 128 tile against 28 - 31 thousand of k
 * loop) but kept in registers and stored a few rows per k step during the NEXT tile of the
 * workgroup, behind that step's operand loads and behind its last MFMA (the matrix core works on
 * while the wave issues them).  Vector memory operations retire in order, so the wait in front of
 * the following step leaves exactly those stores in flight.  Interior tiles
 * with a following tile only; edge tiles and a workgroup's last tile store at once.  fp32 output
 * alone (no int32 output, no residual). */
template <int BM, int BN, int STAGES, int WM, int WN, int EPI, bool TABLE = false, bool DEFER = false>
__global__ __launch_bounds__(WM * WN * 64, (DEFER && BM * BN >= 128 * 128 ? 2 : BM * BN >= 128 * 128 ? 3 : 4)) void bl_gemm_tile256(const uint8_t* __restrict__ packed,
                                                                const int8_t* __restrict__ q,
                                                                const int32_t* __restrict__ rowsum,
                                                                const float* __restrict__ beta,
                                                                const float* __restrict__ scale, int M, int N,
                                                                int K, int tiles_m, int tiles_n, int gm,
                                                                int vgrid, const float* __restrict__ residual,
                                                                int32_t* __restrict__ acc, float* __restrict__ y,
                                                                uint16_t* __restrict__ xb, int* __restrict__ absmax,
                                                                long long* __restrict__ stamps,
                                                                const bl_tile_item* __restrict__ items,
                                                                const int* __restrict__ tile0, int nitems,
                                                                const int* __restrict__ wg_start,
                                                                const int* __restrict__ tile_list) {
    static_assert(!TABLE || EPI == 0, "the table walk has the plain epilogue only");
    static_assert(!DEFER || (EPI == 0 && !TABLE && STAGES == 2), "deferred stores: plain epilogue, two stages");
    static_assert(EPI != 2 || (BN == 128 && WN == 2 && BN / WN / 32 == 2), "the gate epilogue pairs ni = 0 with ni = 1");
    constexpr int NW = WM * WN, THREADS = NW * 64;
    constexpr int G3_BM = BM, G3_A_BYTES = BM * G3_BK;
    constexpr int G3_W_BYTES = BN * G3_BK / 4, G3_STAGE_BYTES = G3_A_BYTES + G3_W_BYTES;
    constexpr int MI = G3_BM / WM / 32, NI = BN / WN / 32;
    constexpr int A_LOADS = G3_A_BYTES / 16 / THREADS;      /* direct loads per thread and stage */
    constexpr int W_LOADS = G3_W_BYTES / 16 / THREADS;
    constexpr int LOADS = A_LOADS + W_LOADS;
    static_assert((STAGES - 2) * LOADS < 64, "vmcnt is a 6-bit count");
    static_assert(THREADS >= BM, "one thread per tile row fetches the row terms");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    /* behind the stages: the per-row terms of the tile in flight (row sum, beta*scale) */
    /* (DEFER: two sets, the second for the tile whose stores are still pending) */
    int* const rs_base = (int*)(smem + STAGES * G3_STAGE_BYTES);
    int* rs_s = rs_base;
    float* cf_s = (float*)(rs_base + G3_BM);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int wm0 = (wave / WN) * (MI * 32), wn0 = (wave % WN) * (NI * 32);
    /* fixed for the launch, or (TABLE) those of the product whose tile is set up next */
    int kb = K / 4;
    int steps = K / G3_BK;
    bool want_cf = EPI != 0 || y != nullptr;            /* the fused epilogues always rescale */
    float bt = (!TABLE && want_cf) ? *beta : 0.0f;
    /* what the epilogue of the tile in flight stores to (TABLE: set when that tile was set up) */
    int eN = N;
    const float* eres = residual;
    int32_t* eacc = acc;
    float* ey = y;
    int nN = N, nsteps = steps;
    const float* nres = residual;
    int32_t* nacc = acc;
    float* ny = y;
    auto load_item = [&](int vb, int& tn) {
        int lo = 0, hi = nitems - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (tile0[mid] <= vb) lo = mid; else hi = mid - 1;
        }
        const bl_tile_item it = items[lo];
        tn = vb - tile0[lo];
        packed = it.packed;
        q = it.q;
        rowsum = it.rowsum;
        scale = it.scale;
        N = nN = it.N;
        K = it.K;
        kb = K / 4;
        nsteps = K / G3_BK;
        nres = it.residual;
        nacc = it.acc;
        ny = it.y;
        want_cf = it.y != nullptr;
        bt = want_cf ? *it.beta : 0.0f;
    };

    /* XCD-aware tile order: workgroup L runs on XCD L%8.  The tile grid is cut
     * into gm x gn = 8 rectangular regions, one per XCD, narrow enough in M that
     * a region's activation panel stays in that XCD's 4 MB L2 while its weight
     * tiles stream through; inside a region the row tiles vary fastest.  The grid is
     * persistent: a workgroup takes virtual blocks vb = blockIdx.x, + gridDim.x, .. (gridDim.x
     * is a multiple of 8, so a workgroup stays on its XCD's region). */
    const int gn = 8 / gm;
    const int rm = (tiles_m + gm - 1) / gm, rn = (tiles_n + gn - 1) / gn;
    auto tile_of = [&](int vb, int& tm, int& tn) {
        const int xcd = vb & 7, idx = vb >> 3;
        tm = (xcd / gn) * rm + idx % rm;
        tn = (xcd % gn) * rn + idx / rm;
        return tm < tiles_m && tn < tiles_n;
    };
    int vend = vgrid;
    if constexpr (TABLE) vend = wg_start[blockIdx.x + 1];
    /* the next virtual block of this workgroup that maps to a real tile, or -1 */
    auto next_tile = [&](int vb, int& tm, int& tn) {
        if constexpr (TABLE) {                      /* vb: position in this workgroup's tile list */
            if (vb >= vend) return -1;
            tm = 0;
            load_item(tile_list[vb], tn);
            return vb;
        }
        for (; vb < vgrid; vb += (int)gridDim.x)
            if (tile_of(vb, tm, tn)) return vb;
        return -1;
    };

    /* per-lane global sources of the direct loads of the tile (tm, tn) */
    const uint8_t* asrc[A_LOADS];
    const uint8_t* wsrc[W_LOADS];
    int row_rs = 0;
    float row_cf = 0.0f;
    auto setup = [&](int tm, int tn) {
        const int m0 = tm * G3_BM, n0 = tn * BN;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
            const int row = (j * NW + wave) * 8 + (lane >> 3);          /* row of the tile */
            const int u = (lane & 7) ^ ((row >> 1) & 7);
            int m = m0 + row;
            if (m >= M) m = M - 1;
            asrc[j] = (const uint8_t*)q + (int64_t)m * K + u * 16;
        }
        const int u = (lane & 1) ^ ((lane >> 4) & 1);
#pragma unroll
        for (int j = 0; j < W_LOADS; ++j) {
            const int trow = (j * NW + wave) * 32 + (lane >> 1);        /* row of the weight tile */
            int n = n0 + trow;
            if (EPI == 2)   /* tile rows [64w, 64w+32) = gate rows, [64w+32, 64w+64) = the matching up rows */
                n = ((trow >> 5) & 1) * (N / 2) + tn * (BN / 2) + (trow >> 6) * 32 + (trow & 31);
            if (n >= N) n = N - 1;
            wsrc[j] = packed + (int64_t)n * kb + u * 16;
        }
        /* the tile's per-row terms travel in two registers until the epilogue (a load there
         * would put a memory round trip between the last MFMA and the first store) */
        if (tid < G3_BM) {
            const int m = m0 + tid;
            row_rs = m < M ? rowsum[m] : 0;
            row_cf = (want_cf && m < M) ? bt * scale[m] : 0.0f;
        }
    };
    auto issue = [&](int kk, int buf) {
        uint8_t* st = smem + buf * G3_STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j)
            __builtin_amdgcn_global_load_lds((bl_gptr)(asrc[j] + (int64_t)kk * G3_BK),
                                             (bl_lptr)(st + (j * NW + wave) * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < W_LOADS; ++j)
            __builtin_amdgcn_global_load_lds((bl_gptr)(wsrc[j] + (int64_t)kk * (G3_BK / 4)),
                                             (bl_lptr)(st + G3_A_BYTES + (j * NW + wave) * 1024), 16, 0, 0);
    };

    /* per-lane LDS read offsets (bytes) inside a stage */
    const int a_row_off = (wm0 + l32) * G3_BK;
    const int a_swz = (l32 >> 1) & 7;
    const int w_off = G3_A_BYTES + ((wn0 + l32) * 2 + (h ^ ((l32 >> 3) & 1))) * 16;

    int tm, tn;
    int vb = next_tile(TABLE ? wg_start[blockIdx.x] : (int)blockIdx.x, tm, tn);
    if (vb < 0) return;
    /* measurement hook: workgroup 0 counts shader clocks and wall-clock ticks over its lifetime
     * (a wave-uniform test, so the counts stay in scalar registers) */
    const bool stamp = stamps != nullptr && blockIdx.x == 0;
    long long c_start = 0, w_start = 0;
    if (stamp) {
        c_start = clock64();
        w_start = wall_clock64();
    }
    setup(tm, tn);
    if constexpr (TABLE) {
        steps = nsteps; eN = nN; eres = nres; eacc = nacc; ey = ny;
    }
    /* STAGES - 1 k steps are in flight ahead of the matrix cores: a k step of one workgroup
     * takes far less time than a load, so the depth, not the tile, hides the latency */
    for (int s0 = 0; s0 < STAGES - 1 && s0 < steps; ++s0) issue(s0, s0);

    /* DEFER: the accumulators of the workgroup's previous tile, where that tile lies and which set
     * of per-row terms is its; cset = the set of the tile in flight */
    bl_v16i P[MI][NI];
    bool have_prev = false;
    int pm0 = 0, pn0 = 0, pset = 0, cset = 0;
    constexpr int RPG = 4;                      /* rows of a lane per store group (2: equal; 1: more groups than k steps at K = 2560, slower) */
    constexpr int GROUPS = MI * 4 * (4 / RPG);  /* store groups of a tile: RPG of the rows 8 vq + 4 h + (0..3) of row block mi */
    constexpr int SPG = RPG * NI;               /* store instructions of a group */
    /* group g of the accumulators A of the tile at (sm0, sn0) -> y; masked: the tile may cross M or N */
    auto emit_rows = [&](const bl_v16i (&A)[MI][NI], const int g, const int sm0, const int sn0, const int set,
                         const bool masked) __attribute__((always_inline)) {
        const int mi = g / 4, vq = g % 4;
        const int* rs_p = rs_base + set * 2 * G3_BM;
        const float* cf_p = (const float*)(rs_p + G3_BM);
        /* (the row is hidden from the compiler here: it would otherwise keep the 64-bit addresses of
         * all 16 * MI * NI stores of a lane in registers across the k loop) */
        int mlb = wm0 + mi * 32 + vq * 8 + h * 4;
        asm volatile("" : "+v"(mlb));
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const int ml = mlb + v4;
            const int m = sm0 + ml;
            const int rs = rs_p[ml];
            const float c = cf_p[ml];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int n = sn0 + wn0 + ni * 32 + l32;
                if (!masked || (m < M && n < eN))
                    __builtin_nontemporal_store((float)(A[mi][ni][vq * 4 + v4] - rs) * c, ey + (int64_t)m * eN + n);
            }
        }
    };

    /* group g of the previous tile, whose finished fp32 values wait in P: one address add and one
     * store per value (32-bit byte offsets from the uniform base: the host sends outputs of 4 GiB
     * or more to the kernel without deferred stores) */
    auto emit_prev = [&](const int g) __attribute__((always_inline)) {
        constexpr int GPQ = 4 / RPG;                     /* groups per block of four rows */
        const int mi = g / (4 * GPQ), vq = (g / GPQ) % 4, v0 = (g % GPQ) * RPG;
        int mlb = wm0 + mi * 32 + vq * 8 + h * 4;
        asm volatile("" : "+v"(mlb));
        const uint32_t bo = ((uint32_t)(pm0 + mlb) * (uint32_t)eN + (uint32_t)(pn0 + wn0 + l32)) * 4u;
#pragma unroll
        for (int v4 = v0; v4 < v0 + RPG; ++v4)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                __builtin_nontemporal_store(__int_as_float(P[mi][ni][vq * 4 + v4]),
                                            (float*)((char*)ey + (size_t)(bo + ((uint32_t)v4 * (uint32_t)eN + ni * 32u) * 4u)));
    };

    while (true) {
        const int m0 = tm * G3_BM, n0 = tn * BN;
        if constexpr (DEFER) {
            rs_s = rs_base + cset * 2 * G3_BM;
            cf_s = (float*)(rs_s + G3_BM);
        }
        bl_v16i C[MI][NI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) C[mi][ni][v] = 0;

        for (int kk = 0; kk < steps; ++kk) {
            /* stage kk must have landed; the stages issued after it may stay in flight */
            const int later = steps - 1 - kk;
            if constexpr (DEFER) {
                /* the SPG stores of the step before were issued behind this stage's loads: they may
                 * stay in flight (vector memory operations retire in order) */
                if (have_prev && kk >= 1 && kk <= GROUPS) BL_WAIT_VM(SPG);
                else BL_WAIT_VM(0);
            } else {
                bl_wait_stages<STAGES - 2, LOADS>(later < STAGES - 2 ? later : STAGES - 2);
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (kk + STAGES - 1 < steps) issue(kk + STAGES - 1, (kk + STAGES - 1) % STAGES);
            const uint8_t* st = smem + (kk % STAGES) * G3_STAGE_BYTES;
            /* operands of sub-step ks+1 are fetched while ks multiplies */
            bl_v4i wq[NI], a[2][MI];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) wq[ni] = *(const bl_v4i*)(st + w_off + ni * 32 * 32);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                a[0][mi] = *(const bl_v4i*)(st + a_row_off + mi * 32 * G3_BK + (((4 * h) ^ a_swz) * 16));
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks < 3) {
                    const int unit = ((4 * h + ks + 1) ^ a_swz) * 16;
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        a[(ks + 1) & 1][mi] = *(const bl_v4i*)(st + a_row_off + mi * 32 * G3_BK + unit);
                }
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const bl_v4i bop = bl_unpack16((uint32_t)wq[ni][ks]);
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        C[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[ks & 1][mi], bop, C[mi][ni], 0, 0, 0);
                }
            }
            /* the pending stores go out behind the step's last MFMA: the matrix core works on while
             * the wave issues them */
            if constexpr (DEFER) {
                if (have_prev && kk < GROUPS) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int g = 0; g < GROUPS; ++g)
                        if (kk == g) emit_prev(g);
                }
            }
        }

        /* Epilogue.  The per-row terms go through LDS once: a load per output row inside the
         * store loop would serialise on latency.  Every wave is past its last stage read after
         * the barrier, so the first stages of this workgroup's NEXT tile are requested here and
         * travel while this tile is stored. */
        if constexpr (DEFER) {
            if (have_prev) {
#pragma unroll
                for (int g = 0; g < GROUPS; ++g)
                    if (g >= steps) emit_prev(g);
                have_prev = false;
            }
        }
        bl_mfma_fence();
        if (tid < G3_BM) {
            rs_s[tid] = row_rs;
            cf_s[tid] = row_cf;
        }
        /* these LDS writes must have been performed before any wave passes the barrier (a raw
         * s_barrier does not wait for them) */
        BL_WAIT_LGKM0();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        int tm2 = 0, tn2 = 0;
        const int vb2 = next_tile(vb + (TABLE ? 1 : (int)gridDim.x), tm2, tn2);
        if (vb2 >= 0) {
            setup(tm2, tn2);
            for (int s0 = 0; s0 < STAGES - 1 && s0 < (TABLE ? nsteps : steps); ++s0) issue(s0, s0);
        }
        if constexpr (DEFER) {
            if (vb2 >= 0 && m0 + G3_BM <= M && n0 + BN <= eN) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int ml = wm0 + mi * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
                        const int rs = rs_s[ml];
                        const float c = cf_s[ml];
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) P[mi][ni][v] = __float_as_int((float)(C[mi][ni][v] - rs) * c);
                    }
                pm0 = m0;
                pn0 = n0;
                pset = cset;
                have_prev = true;
            } else {
#pragma unroll
                for (int g = 0; g < MI * 4; ++g) emit_rows(C, g, m0, n0, cset, true);
            }
            cset ^= 1;
        } else if constexpr (EPI == 0) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                /* the residual values of four rows first, then their stores back to back: a load
                 * between two stores would make each store wait for the one before it */
                float rres[4][NI];
                if (eres && ey) {
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        const int m = m0 + wm0 + mi * 32 + vq * 8 + h * 4 + v4;
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) {
                            const int n = n0 + wn0 + ni * 32 + l32;
                            rres[v4][ni] = (m < M && n < eN) ? eres[(int64_t)m * eN + n] : 0.0f;
                        }
                    }
                }
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const int v = vq * 4 + v4;
                    const int ml = wm0 + mi * 32 + vq * 8 + h * 4 + v4;
                    const int m = m0 + ml;
                    if (m < M) {
                        const int rs = rs_s[ml];
                        const float c = cf_s[ml];
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) {
                            const int n = n0 + wn0 + ni * 32 + l32;
                            if (n < eN) {
                                const int val = C[mi][ni][v] - rs;
                                if (eacc) eacc[(int64_t)m * eN + n] = val;
                                if (ey) {
                                    const float t = (float)val * c;
                                    const float out = eres ? rres[v4][ni] + t : t;
                                    __builtin_nontemporal_store(out, ey + (int64_t)m * eN + n);
                                }
                            }
                        }
                    }
                }
            }
        } else {
            /* fused producer epilogue: glue value t, its bf16 narrowing (the next BitLinear's input
             * before quantisation) and the row maximum of |bf16(t)|: over the lane's columns, then over
             * the 32 lanes of a half wave (butterfly), then one atomic max per row on the float bits
             * (non-negative floats order like integers, so the result does not depend on the order) */
            const int NOUT = EPI == 2 ? N / 2 : N;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    float rres[4][NI];
                    if (EPI == 1) {
#pragma unroll
                        for (int v4 = 0; v4 < 4; ++v4) {
                            const int m = m0 + wm0 + mi * 32 + vq * 8 + h * 4 + v4;
#pragma unroll
                            for (int ni = 0; ni < NI; ++ni) {
                                const int n = n0 + wn0 + ni * 32 + l32;
                                rres[v4][ni] = (m < M && n < N) ? residual[(int64_t)m * N + n] : 0.0f;
                            }
                        }
                    }
                    float rowmax[4];
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        const int v = vq * 4 + v4;
                        const int ml = wm0 + mi * 32 + vq * 8 + h * 4 + v4;
                        const int m = m0 + ml;
                        float mx = 0.0f;
                        if (m < M) {
                            const int rs = rs_s[ml];
                            const float c = cf_s[ml];
                            if (EPI == 1) {
#pragma unroll
                                for (int ni = 0; ni < NI; ++ni) {
                                    const int n = n0 + wn0 + ni * 32 + l32;
                                    if (n < N) {
                                        const int val = C[mi][ni][v] - rs;
                                        if (acc) acc[(int64_t)m * N + n] = val;
                                        const float t = (float)val * c;
                                        const float o = rres[v4][ni] + t;
                                        if (y) __builtin_nontemporal_store(o, y + (int64_t)m * N + n);
                                        const uint32_t bits = bl_f32_to_bf16(o);
                                        xb[(int64_t)m * NOUT + n] = (uint16_t)bits;
                                        mx = fmaxf(mx, fabsf(bl_bf16_to_f32(bits)));
                                    }
                                }
                            } else {
                                const int j = tn * (BN / 2) + wn0 / 2 + l32;     /* column of the gated output */
                                if (j < NOUT) {
                                    const int vg = C[mi][0][v] - rs, vu = C[mi][NI - 1][v] - rs;
                                    if (acc) {
                                        acc[(int64_t)m * N + j] = vg;
                                        acc[(int64_t)m * N + NOUT + j] = vu;
                                    }
                                    const float g = (float)vg * c, u = (float)vu * c;
                                    const float r = fmaxf(g, 0.0f);
                                    const float r2 = r * r;
                                    const float o = r2 * u;
                                    if (y) __builtin_nontemporal_store(o, y + (int64_t)m * NOUT + j);
                                    const uint32_t bits = bl_f32_to_bf16(o);
                                    xb[(int64_t)m * NOUT + j] = (uint16_t)bits;
                                    mx = fmaxf(mx, fabsf(bl_bf16_to_f32(bits)));
                                }
                            }
                        }
                        rowmax[v4] = mx;
                    }
#pragma unroll
                    for (int off = 1; off < 32; off <<= 1)
#pragma unroll
                        for (int v4 = 0; v4 < 4; ++v4) rowmax[v4] = fmaxf(rowmax[v4], __shfl_xor(rowmax[v4], off));
                    if (l32 == 0) {
#pragma unroll
                        for (int v4 = 0; v4 < 4; ++v4) {
                            const int m = m0 + wm0 + mi * 32 + vq * 8 + h * 4 + v4;
                            if (m < M) atomicMax(absmax + m, __float_as_int(rowmax[v4]));
                        }
                    }
                }
        }
        if (vb2 < 0) {
            if (stamp && tid == 0) {
                stamps[0] = clock64() - c_start;
                stamps[1] = wall_clock64() - w_start;
            }
            break;
        }
        vb = vb2;
        tm = tm2;
        tn = tn2;
        if constexpr (TABLE) {
            steps = nsteps; eN = nN; eres = nres; eacc = nacc; ey = ny;
        }
        /* the next tile's epilogue rewrites rs_s / cf_s only after its own k loop, whose barriers
         * every wave passes after it has finished the reads above */
    }
}

/* Outputs of the fused producer epilogues (device pointers; see bl_gemm_tile256). */
struct bl_epi_args {
    uint16_t* xb;
    int* absmax;
};

template <int BM, int BN, int STAGES, int WM, int WN, int EPI = 0, bool DEFER = false>
static bl_status launch_tile256_t(const uint8_t* packed, const float* beta, const int8_t* q, const float* scale,
                                  const int32_t* rowsum, int M, int N, int K, const float* residual,
                                  int32_t* acc, float* y, hipStream_t st, bl_epi_args ep = bl_epi_args{nullptr, nullptr}) {
    constexpr int G3_BM = BM;
    constexpr int lds = STAGES * (BM * G3_BK + BN * G3_BK / 4) + BM * 8 * (DEFER ? 2 : 1);
    auto kern = bl_gemm_tile256<BM, BN, STAGES, WM, WN, EPI, false, DEFER>;
    static std::atomic<bool> attr_set;
    if (!attr_set.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return BL_ERR_HIP;
        attr_set.store(true, std::memory_order_release);
    }
    /* the gate epilogue's tile holds 64 gate rows and the 64 matching up rows: N/2 / 64 column tiles */
    const int tiles_m = (M + G3_BM - 1) / G3_BM, tiles_n = EPI == 2 ? (N / 2 + BN / 2 - 1) / (BN / 2) : (N + BN - 1) / BN;
    /* rows of activations per XCD region: at most ~1.5 MB of int8 (measured, medians of six
     * interleaved rounds at M = 2048: +7 % on the 13824-wide shape against whole-M regions,
     * equal on the others) */
    int gm = 1;
    while (gm < 8 && (int64_t)((tiles_m + gm - 1) / gm) * BM * K > (3 << 19)) gm *= 2;
    const int gn = 8 / gm;
    const int vgrid = 8 * ((tiles_m + gm - 1) / gm) * ((tiles_n + gn - 1) / gn);
    /* persistent grid: what is resident at once (a multiple of 8 keeps a workgroup on its XCD's region) */
    static std::atomic<int> resident{0};
    int blocks = resident.load(std::memory_order_acquire);
    if (blocks == 0) {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)kern, WM * WN * 64, lds) != hipSuccess ||
            cus < 1 || per_cu < 1)
            return BL_ERR_HIP;
        blocks = cus * per_cu / 8 * 8;
        if (blocks < 8) blocks = 8;
        resident.store(blocks, std::memory_order_release);
    }
    if (blocks > vgrid) blocks = vgrid;
    kern<<<blocks, WM * WN * 64, lds, st>>>(packed, q, rowsum, beta, scale, M, N, K, tiles_m, tiles_n, gm, vgrid,
                                            residual, acc, y, ep.xb, ep.absmax, (long long*)bl_clock_stamps(), nullptr, nullptr, 0, nullptr, nullptr);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

/* Table walk (batched decode of a stack, more than 48 tokens): 64 x 128 tiles, one launch over
 * every tile of every product.  items / tile0: device arrays of `nitems` entries (tile0 ascending,
 * tile0[0] = 0); total_tiles = tiles of the whole table; M <= 64 tokens, the same for every
 * product.  Workgroup b takes the tiles tile_list[wg_start[b] .. wg_start[b+1]) (device arrays
 * of blocks + 1 and total_tiles entries: the host balances the k steps over the workgroups).
 * bl_gemm_table_blocks: the persistent grid (resident workgroups), 0 on error. */
static constexpr int TABLE_LDS = 2 * (64 * G3_BK + 128 * G3_BK / 4) + 64 * 8;
static std::atomic<int> g_table_blocks{0};

int bl_gemm_table_blocks(void) {
    int blocks = g_table_blocks.load(std::memory_order_acquire);
    if (blocks > 0) return blocks;
    auto kern = bl_gemm_tile256<64, 128, 2, 1, 4, 0, true>;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TABLE_LDS) != hipSuccess ||
        hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)kern, 256, TABLE_LDS) != hipSuccess ||
        cus < 1 || per_cu < 1)
        return 0;
    blocks = cus * per_cu;
    g_table_blocks.store(blocks, std::memory_order_release);
    return blocks;
}

bl_status bl_gemm_table_launch(const bl_tile_item* items, const int* tile0, int nitems, int total_tiles, int M,
                               int blocks, const int* wg_start, const int* tile_list, bl_stream s) {
    hipStream_t st = (hipStream_t)s;
    if (g_table_blocks.load(std::memory_order_acquire) == 0) return BL_ERR_VALUE;   /* no table was built in this process */
    bl_gemm_tile256<64, 128, 2, 1, 4, 0, true><<<blocks, 256, TABLE_LDS, st>>>(
        nullptr, nullptr, nullptr, nullptr, nullptr, M, 0, G3_BK, 1, 0, 1, total_tiles, nullptr, nullptr, nullptr, nullptr,
        nullptr, nullptr, items, tile0, nitems, wg_start, tile_list);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
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
                           const float* residual, int32_t* acc, float* y, void* workspace, hipStream_t st) {
    if (!rowsum) {
        if (!workspace) return BL_ERR_WORKSPACE;
        if (!bl_aligned(workspace, 4)) return BL_ERR_ALIGN;
        int32_t* rs = (int32_t*)workspace;
        bl_rowsum_kernel<<<(unsigned)((M + 3) / 4), 256, 0, st>>>(q, (int)M, (int)K, rs);
        rowsum = rs;
    }
    /* Tile choice.  Measured on MI355X at M = 2048 on the four 2B-layer shapes: 128x128 tiles,
     * k step 128, two LDS stages filled by direct global->LDS loads, XCD-aware tile order, three
     * workgroups per CU: about 1450 TOPS over the layer against 1310 for the register-staged
     * 128x128 kernel.  Also measured and dropped (no longer in the library): 256x256 tiles with
     * 2x2 / 2x4 / 4x2 waves and 256x128 (0.9 - 1.1 POP/s), a three-stage 128x128 and 4- or 6-stage
     * pipelines (what hides the load latency is the number of workgroups per CU, not the depth),
     * 64x256 (equal within noise).  When the problem has at most ~1.5 tiles of 128x128 per CU,
     * 64x128 tiles balance better: +17..21 % on the N = 2560 shapes at M = 2048, +22..27 % on every
     * small shape at M = 1024, equal at 480 tiles and slower on the wide shape.  Both need layout 1
     * and K % 128 == 0; other inputs use the register-staged kernel, which permutes the activation
     * bytes for layout 0. */
    const int m = (int)M, n = (int)N, k = (int)K;
    if (layout == 1 && k % G3_BK == 0) {
        if ((int64_t)((m + 127) / 128) * ((n + 127) / 128) <= 400)
            return launch_tile256_t<64, 128, 2, 1, 4>(packed, beta, q, scale, rowsum, m, n, k, residual, acc, y, st);
        /* fp32 output alone: the stores of a tile travel during the workgroup's next tile (measured at
         * M = 2048 / 8192: the 13824-wide shape 77 - 80 us against 86 - 90, 297 - 308 against 317 - 327;
         * the 64 x 128 kernel with deferred stores loses: it has under one tile per workgroup on the
         * shapes it serves) */
        if (!acc && !residual && (int64_t)m * n < ((int64_t)1 << 30))
            return launch_tile256_t<128, 128, 2, 2, 2, 0, true>(packed, beta, q, scale, rowsum, m, n, k, residual, acc, y, st);
        return launch_tile256_t<128, 128, 2, 2, 2>(packed, beta, q, scale, rowsum, m, n, k, residual, acc, y, st);
    }
    if (k % 128 == 0)
        return launch_gemm<128, 128, 128, 2>(packed, beta, layout, q, scale, rowsum, m, n, k, residual, acc, y, st);
    return launch_gemm<128, 128, 64, 2>(packed, beta, layout, q, scale, rowsum, m, n, k, residual, acc, y, st);
}

extern "C" bl_status bl_gemm_w158a8_res(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                                        const float* scale, const int32_t* rowsum, int64_t M, int64_t N, int64_t K,
                                        const float* residual, int32_t* acc, float* y, void* workspace,
                                        bl_stream s) {
    if (!packed || !beta || !q) return BL_ERR_NULL;
    if (!acc && !y) return BL_ERR_NULL;
    if (y && !scale) return BL_ERR_NULL;
    if (M < 1 || M > BL_MAX_DIM || !bl_shape_ok(N, K)) return BL_ERR_SHAPE;
    if (layout != BL_LAYOUT_ROWMAJOR && layout != BL_LAYOUT_K16) return BL_ERR_LAYOUT;
    if (!bl_aligned(packed, 16) || !bl_aligned(q, 16) || !bl_aligned(acc, 4) || !bl_aligned(y, 4) ||
        !bl_aligned(scale, 4) || !bl_aligned(beta, 4) || !bl_aligned(rowsum, 4) || !bl_aligned(residual, 4))
        return BL_ERR_ALIGN;
    return bl_gemm_dispatch(packed, beta, layout, q, scale, rowsum, M, N, bl_kpad(K), residual, acc, y, workspace,
                            (hipStream_t)s);
}

extern "C" bl_status bl_gemm_w158a8(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                                    const float* scale, const int32_t* rowsum, int64_t M, int64_t N, int64_t K,
                                    int32_t* acc, float* y, void* workspace, bl_stream s) {
    return bl_gemm_w158a8_res(packed, beta, layout, q, scale, rowsum, M, N, K, nullptr, acc, y, workspace, s);
}

/* Prefill product with a fused producer epilogue (see bl_gemm_tile256, EPI = 1 and 2). */
extern "C" bl_status bl_gemm_w158a8_fused(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                                          const float* scale, const int32_t* rowsum, int64_t M, int64_t N, int64_t K,
                                          const bl_gemm_epilogue* ep, int32_t* acc, bl_stream s) {
    if (!packed || !beta || !q || !scale || !rowsum || !ep) return BL_ERR_NULL;
    if (!ep->x_bf16 || !ep->absmax) return BL_ERR_NULL;
    if (ep->kind != BL_EPI_RESIDUAL && ep->kind != BL_EPI_RELU2_GATE) return BL_ERR_VALUE;
    if (ep->kind == BL_EPI_RESIDUAL && !ep->residual) return BL_ERR_NULL;
    if (M < 1 || M > BL_MAX_DIM || !bl_shape_ok(N, K) || K % G3_BK != 0 || N % 4 != 0) return BL_ERR_SHAPE;
    if (ep->kind == BL_EPI_RELU2_GATE && N % 128 != 0) return BL_ERR_SHAPE;   /* N/2 gate columns in tiles of 64 */
    if (layout != BL_LAYOUT_K16) return BL_ERR_LAYOUT;
    if (!bl_aligned(packed, 16) || !bl_aligned(q, 16) || !bl_aligned(acc, 4) || !bl_aligned(ep->y, 4) ||
        !bl_aligned(scale, 4) || !bl_aligned(beta, 4) || !bl_aligned(rowsum, 4) || !bl_aligned(ep->residual, 4) ||
        !bl_aligned(ep->x_bf16, 2) || !bl_aligned(ep->absmax, 4))
        return BL_ERR_ALIGN;
    const bl_epi_args ea = {ep->x_bf16, (int*)ep->absmax};
    hipStream_t st = (hipStream_t)s;
    if (ep->kind == BL_EPI_RESIDUAL)
        return launch_tile256_t<128, 128, 2, 2, 2, 1>(packed, beta, q, scale, rowsum, (int)M, (int)N, (int)K,
                                                      ep->residual, acc, ep->y, st, ea);
    return launch_tile256_t<128, 128, 2, 2, 2, 2>(packed, beta, q, scale, rowsum, (int)M, (int)N, (int)K, nullptr, acc,
                                                  ep->y, st, ea);
}

/* ---- entry point that allocates nothing ---------------------------------------------------
 * bl_gemm_w158a8 needs device scratch for the row sums sum_k q[m][k] when the caller brings
 * none.  Here that scratch is a static device array: every GPU the library runs on holds its
 * own copy, at its own address, until the process ends.  In host code the array's name is only
 * a stand-in: the device address comes from hipGetSymbolAddress, once per device, and that
 * pointer is what the kernels receive. */
#define BL_NOALLOC_MAX_DEVICES 64
static __device__ __align__(256) int32_t scratch[BL_NOALLOC_MAX_M];
static std::atomic<int32_t*> bl_scratch_ptr[BL_NOALLOC_MAX_DEVICES];

static bl_status bl_scratch_for_current_device(int32_t** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= BL_NOALLOC_MAX_DEVICES) return BL_ERR_HIP;
    int32_t* p = bl_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        /* two threads racing here both obtain the same address: the symbol has one copy per device */
        void* sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return BL_ERR_HIP;
        p = (int32_t*)sym;
        bl_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return BL_OK;
}

extern "C" bl_status bl_gemm_w158a8_noalloc(const uint8_t* packed, const float* beta, int layout, const int8_t* q,
                                            const float* scale, int64_t M, int64_t N, int64_t K, int32_t* acc,
                                            float* y, bl_stream s) {
    if (!packed || !beta || !q) return BL_ERR_NULL;
    if (!acc && !y) return BL_ERR_NULL;
    if (y && !scale) return BL_ERR_NULL;
    if (M < 1 || M > BL_NOALLOC_MAX_M || !bl_shape_ok(N, K)) return BL_ERR_SHAPE;
    if (layout != BL_LAYOUT_ROWMAJOR && layout != BL_LAYOUT_K16) return BL_ERR_LAYOUT;
    if (!bl_aligned(packed, 16) || !bl_aligned(q, 16) || !bl_aligned(acc, 4) || !bl_aligned(y, 4) ||
        !bl_aligned(scale, 4) || !bl_aligned(beta, 4))
        return BL_ERR_ALIGN;
    int32_t* rs = nullptr;
    const bl_status st = bl_scratch_for_current_device(&rs);
    if (st != BL_OK) return st;
    /* the row-sum kernel overwrites entries 0..M-1 and nothing reads beyond them, so what an
     * earlier (larger) call left behind needs no clearing */
    return bl_gemm_dispatch(packed, beta, layout, q, scale, nullptr, M, N, bl_kpad(K), nullptr, acc, y, rs, (hipStream_t)s);
}
