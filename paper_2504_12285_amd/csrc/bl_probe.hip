/* Measurement aids: the two achievable roofs the BitLinear kernels are priced against beside
 * the datasheet peaks.  bl_probe_stream_read is a plain 16-byte-per-lane streaming read of a
 * large buffer (what the memory system delivers to a kernel that does nothing else);
 * bl_probe_mfma_i8 is a register-resident loop of v_mfma_i32_32x32x32_i8 (what the matrix
 * cores deliver with no operand traffic at all).  Neither is part of the product path. */
#include "bl_device.h"
#include "bl_host.h"

typedef bl_v4i __attribute__((address_space(1))) bl_pgv4i;

/* The buffer is cut into one contiguous slice per workgroup (as the streaming decode kernel
 * cuts its table); inside a slice wave w reads blocks w, w + 4, .. of 8 KiB: eight 1 KiB wave-wide
 * loads in flight per wave.  The XOR of everything read goes to sink[] only if it equals a value
 * that random data never produces in practice, so the loads cannot be removed. */
__global__ __launch_bounds__(256) void bl_probe_read_kernel(const bl_v4i* __restrict__ buf, int64_t n16,
                                                             int32_t* __restrict__ sink) {
    const bl_pgv4i* p = (const bl_pgv4i*)buf;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t nblk = n16 / 512;                       /* whole 8 KiB blocks */
    const int64_t b0 = nblk * blockIdx.x / gridDim.x, b1 = nblk * (blockIdx.x + 1) / gridDim.x;
    bl_v4i x = {0, 0, 0, 0};
    for (int64_t b = b0 + w; b < b1; b += 4) {
        bl_v4i v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(p + b * 512 + j * 64 + lane);
#pragma unroll
        for (int j = 0; j < 8; ++j) x ^= v[j];
    }
    /* the tail beyond the last whole block */
    for (int64_t i = nblk * 512 + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
        x ^= __builtin_nontemporal_load(p + i);
    const int r = x[0] ^ x[1] ^ x[2] ^ x[3];
    if (r == 0x5EEDF00D) sink[threadIdx.x & 63] = r;
}

/* The write side: every lane stores fp32 values with the prefill epilogue's pattern (a wave-wide
 * dword store = 32 consecutive floats of each of two rows of a row-major [rows][cols] matrix, 64
 * such stores per lane and 64 x 64 tile, non-temporal), the matrix cut into one run of tiles per
 * workgroup, and nothing else: what the memory system takes when every workgroup of a launch
 * stores its tile at the same time. */
__global__ __launch_bounds__(256) void bl_probe_write_kernel(float* __restrict__ buf, int rows, int cols) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int tiles_n = cols / 128, tiles = (rows / 128) * tiles_n;
    for (int t = blockIdx.x; t < tiles; t += gridDim.x) {
        const int m0 = (t / tiles_n) * 128 + (w >> 1) * 64, n0 = (t % tiles_n) * 128 + (w & 1) * 64;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + mi * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    __builtin_nontemporal_store((float)(m + v), buf + (int64_t)m * cols + n0 + ni * 32 + l32);
            }
    }
}

#ifdef BL_PROBE_EXPERIMENTS
/* experiment: the access pattern of the decode kernel (8 lanes per 640-byte row, 8 rows per load) */
__global__ __launch_bounds__(256) void bl_probe_read_rows(const bl_v4i* __restrict__ buf, int64_t n16,
                                                           int32_t* __restrict__ sink, int mode) {
    const bl_pgv4i* p = (const bl_pgv4i*)buf;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t nblk = n16 / 320;                       /* units of 8 rows x 40 chunks */
    const int64_t b0 = nblk * blockIdx.x / gridDim.x, b1 = nblk * (blockIdx.x + 1) / gridDim.x;
    const int r = lane >> 3, g = lane & 7;
    bl_v4i x = {0, 0, 0, 0};
    for (int64_t b = b0 + w; b < b1; b += 4) {
        bl_v4i v[5];
#pragma unroll
        for (int j = 0; j < 5; ++j)
            v[j] = __builtin_nontemporal_load(p + b * 320 + (mode == 0 ? r * 40 + g + 8 * j : j * 64 + lane));
#pragma unroll
        for (int j = 0; j < 5; ++j) x ^= v[j];
    }
    const int rr = x[0] ^ x[1] ^ x[2] ^ x[3];
    if (rr == 0x5EEDF00D) sink[threadIdx.x & 63] = rr;
}
extern "C" int bl_probe_rows(const void* buf, size_t bytes, int per_cu, int mode, int32_t* sink, void* s) {
    int dev = 0, cus = 0;
    hipGetDevice(&dev);
    hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    bl_probe_read_rows<<<cus * per_cu, 256, 0, (hipStream_t)s>>>((const bl_v4i*)buf, (int64_t)(bytes / 16), sink, mode);
    return (int)hipGetLastError();
}
#endif

/* Four independent accumulator chains per wave, operands in registers: constants made from the
 * lane number, or (operands != NULL) 32 bytes per lane read once from memory, e.g. random int8
 * values: the rate of this loop depends on the switching activity of its operands, because the
 * chip lowers its clock under the power such a loop draws.  stamps (or NULL) receives what
 * workgroup 0 counted: shader clocks and ticks of the constant-rate wall clock. */
__global__ __launch_bounds__(256) void bl_probe_mfma_kernel(int iters, const bl_v4i* __restrict__ operands,
                                                             long long* __restrict__ stamps,
                                                             int32_t* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    bl_v4i a = {lane * 0x01010101, (lane + 3) * 0x01010101, (lane ^ 21) * 0x01010101, (lane + 9) * 0x01010101};
    bl_v4i b = {0x01020001, 0x00010201, 0x02000102, 0x01010200};
    if (operands) {
        a = operands[(blockIdx.x & 7) * 512 + threadIdx.x * 2];
        b = operands[(blockIdx.x & 7) * 512 + threadIdx.x * 2 + 1];
    }
    const bool stamp = stamps != nullptr && blockIdx.x == 0;          /* uniform: the counters stay scalar */
    long long c_start = 0, w_start = 0;
    if (stamp) {
        c_start = clock64();
        w_start = wall_clock64();
    }
    bl_v16i c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, a, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, b, c3, 0, 0, 0);
    }
    bl_mfma_fence();
    int r = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) r ^= c0[j] ^ c1[j] ^ c2[j] ^ c3[j];
    if (r == 0x5EEDF00D) sink[lane] = r;
    if (stamp && threadIdx.x == 0) {
        stamps[0] = clock64() - c_start;
        stamps[1] = wall_clock64() - w_start;
    }
}

static int probe_grid(int per_cu) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return 0;
    return cus * per_cu;
}

extern "C" bl_status bl_probe_stream_read(const void* buf, size_t bytes, int workgroups_per_cu, int32_t* sink,
                                          bl_stream s) {
    if (!buf || !sink) return BL_ERR_NULL;
    if (bytes < 16 || bytes % 16) return BL_ERR_SHAPE;
    if (!bl_aligned(buf, 16) || !bl_aligned(sink, 4)) return BL_ERR_ALIGN;
    if (workgroups_per_cu < 0 || workgroups_per_cu > 8) return BL_ERR_SHAPE;
    const int blocks = probe_grid(workgroups_per_cu ? workgroups_per_cu : 8);
    if (blocks < 1) return BL_ERR_HIP;
    bl_probe_read_kernel<<<blocks, 256, 0, (hipStream_t)s>>>((const bl_v4i*)buf, (int64_t)(bytes / 16), sink);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

extern "C" bl_status bl_probe_stream_write(float* buf, int64_t rows, int64_t cols, int workgroups_per_cu, bl_stream s) {
    if (!buf) return BL_ERR_NULL;
    if (rows < 128 || cols < 128 || rows % 128 || cols % 128 || rows > (1 << 24) || cols > (1 << 24)) return BL_ERR_SHAPE;
    if (!bl_aligned(buf, 4)) return BL_ERR_ALIGN;
    if (workgroups_per_cu < 0 || workgroups_per_cu > 8) return BL_ERR_SHAPE;
    const int blocks = probe_grid(workgroups_per_cu ? workgroups_per_cu : 3);
    if (blocks < 1) return BL_ERR_HIP;
    bl_probe_write_kernel<<<blocks, 256, 0, (hipStream_t)s>>>(buf, (int)rows, (int)cols);
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

extern "C" bl_status bl_probe_mfma_i8_ex(int iters, const void* operands, int64_t* stamps, int32_t* sink, double* ops,
                                         bl_stream s) {
    if (!sink) return BL_ERR_NULL;
    if (iters < 1 || iters > (1 << 24)) return BL_ERR_SHAPE;
    if (!bl_aligned(sink, 4) || !bl_aligned(operands, 16) || !bl_aligned(stamps, 8)) return BL_ERR_ALIGN;
    const int blocks = probe_grid(2);
    if (blocks < 1) return BL_ERR_HIP;
    bl_probe_mfma_kernel<<<blocks, 256, 0, (hipStream_t)s>>>(iters, (const bl_v4i*)operands, (long long*)stamps, sink);
    if (ops) *ops = (double)blocks * 4.0 * iters * 4.0 * 2.0 * 32.0 * 32.0 * 32.0;
    return hipGetLastError() == hipSuccess ? BL_OK : BL_ERR_HIP;
}

extern "C" bl_status bl_probe_mfma_i8(int iters, int32_t* sink, double* ops, bl_stream s) {
    return bl_probe_mfma_i8_ex(iters, nullptr, nullptr, sink, ops, s);
}

extern "C" int bl_probe_wall_clock_khz(void) {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess)
        return 0;
    return khz;
}
