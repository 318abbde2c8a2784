/*
 * Seeded synthetic inputs for BitLinear experiments: latent fp32 weights and
 * bf16 activations.  This file holds NO arithmetic of the method under test
 * (no quantiser, no packing, no matmul); it only draws numbers.  Both the CPU
 * oracle's tests and the GPU path's tests consume its output as plain data.
 *
 * Generator: counter based.  Element i of stream (seed, stream_id) depends on
 * (seed, stream_id, i) only, so any slice can be produced independently and in
 * parallel with identical results.
 *   key  = mix(mix(seed) ^ stream_id)
 *   r1   = mix(key ^ 2i) ; r2 = mix(key ^ (2i+1))         (SplitMix64 finaliser)
 *   u1   = ((r1 >> 11) + 1) * 2^-53  in (0,1] ; u2 = (r2 >> 11) * 2^-53 in [0,1)
 *   z    = sqrt(-2 ln u1) * cos(2 pi u2)                   (Box-Muller, fp64)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint64_t stream_key(uint64_t seed, uint64_t stream_id) {
    return mix64(mix64(seed) ^ stream_id);
}

static inline double std_normal(uint64_t key, uint64_t i) {
    const uint64_t r1 = mix64(key ^ (2 * i));
    const uint64_t r2 = mix64(key ^ (2 * i + 1));
    const double u1 = (double)((r1 >> 11) + 1) * 0x1.0p-53;
    const double u2 = (double)(r2 >> 11) * 0x1.0p-53;
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
}

/* fp32 -> bf16 bit pattern, round to nearest even (finite inputs only). */
static inline uint16_t f32_to_bf16_bits(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* out[i] = (float)(sigma * z_i), i in [first, first+n). */
void synth_normal_f32(uint64_t seed, uint64_t stream_id, int64_t first, int64_t n,
                      double sigma, float* out) {
    const uint64_t key = stream_key(seed, stream_id);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        out[i] = (float)(sigma * std_normal(key, (uint64_t)(first + i)));
}

/* The first n_out entries of a seeded Fisher-Yates shuffle of 0..K-1. */
void synth_outlier_channels(uint64_t seed, uint64_t stream_id, int64_t K, int64_t n_out,
                            int32_t* out) {
    const uint64_t key = stream_key(seed, stream_id ^ 0x07113Eull);
    int32_t* perm = (int32_t*)malloc((size_t)K * sizeof(int32_t));
    for (int64_t i = 0; i < K; ++i) perm[i] = (int32_t)i;
    for (int64_t i = 0; i < n_out && i < K - 1; ++i) {
        const uint64_t j = (uint64_t)i + mix64(key ^ (uint64_t)i) % (uint64_t)(K - i);
        const int32_t t = perm[i]; perm[i] = perm[j]; perm[j] = t;
    }
    for (int64_t i = 0; i < n_out; ++i) out[i] = perm[i];
    free(perm);
}

/* bf16 activations [M][K]: z ~ N(0,1) in fp32; channels listed in `outliers`
 * multiplied by outlier_mul (fp32); if relu2 != 0 the value becomes
 * max(v,0)^2 (fp32); then narrowed to bf16.  Rows [row0, row0+M) of the stream. */
void synth_activations_bf16(uint64_t seed, uint64_t stream_id, int64_t row0, int64_t M,
                            int64_t K, const int32_t* outliers, int64_t n_out,
                            float outlier_mul, int relu2, uint16_t* out) {
    const uint64_t key = stream_key(seed, stream_id);
    float* mul = (float*)malloc((size_t)K * sizeof(float));
    for (int64_t k = 0; k < K; ++k) mul[k] = 1.0f;
    for (int64_t i = 0; i < n_out; ++i) mul[outliers[i]] = outlier_mul;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t k = 0; k < K; ++k) {
            const uint64_t idx = (uint64_t)((row0 + m) * K + k);
            float v = (float)std_normal(key, idx) * mul[k];
            if (relu2) { v = v > 0.0f ? v : 0.0f; v = v * v; }
            out[m * K + k] = f32_to_bf16_bits(v);
        }
    }
    free(mul);
}

/* Uniform integers in [lo, hi] (inclusive) as int8: raw quantised inputs for
 * tests that bypass the quantiser. */
void synth_uniform_i8(uint64_t seed, uint64_t stream_id, int64_t n, int lo, int hi, int8_t* out) {
    const uint64_t key = stream_key(seed, stream_id);
    const uint64_t span = (uint64_t)(hi - lo + 1);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        out[i] = (int8_t)(lo + (int)(mix64(key ^ (uint64_t)i) % span));
}
