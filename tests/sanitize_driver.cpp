/* Sanitizer run of the CPU-side code (AddressSanitizer + UndefinedBehaviorSanitizer, host only):
 * the oracle's functions on exactly-sized heap buffers over shapes with tails, and the library's
 * host-only entry points.  Built and run by tests/test_sanitizers.py; exits 0 when nothing is
 * reported.  Checks a few invariants on the way so that the calls cannot be optimised away. */
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "bitlinear.h"

extern "C" {
float orc_absmean_beta(const float* W, int64_t N, int64_t K, double* mean64);
void orc_ternarize(const float* W, int64_t N, int64_t K, float beta, int8_t* Wt);
int orc_pack(const int8_t* Wt, int64_t N, int64_t K, int layout, uint8_t* packed);
int64_t orc_unpack(const uint8_t* packed, int64_t N, int64_t K, int layout, int8_t* Wt);
void orc_quant_act(const uint16_t* X, int64_t M, int64_t K, int8_t* q, float* scale, int32_t* rowsum);
void orc_matmul_i32(const int8_t* q, const int8_t* Wt, int64_t M, int64_t N, int64_t K, int32_t* acc);
void orc_matmul_i32_sampled(const int8_t* q, const int8_t* Wt, int64_t N, int64_t K, const int64_t* ms,
                            const int64_t* ns, int64_t count, int32_t* out);
void orc_rescale(const int32_t* acc, float beta, const float* scale, int64_t M, int64_t N, float* y);
void orc_f32_to_bf16(const float* x, int64_t n, uint16_t* out);
void orc_chain_attn_stub(const float* qkv, int64_t M, int n_q, int n_kv, int hd, uint16_t* a);
void orc_chain_residual(const float* x, const float* y, int64_t n, float* h);
void orc_chain_relu2_gate(const float* gu, int64_t M, int64_t F, uint16_t* f);
void orc_rmsnorm_rows(const float* t, int64_t M, int64_t K, const float* gain, float eps, uint16_t* out, double* r64);
void orc_chain_attn_f32(const float* qkv, int64_t M, int n_q, int n_kv, int hd, float* a);
void orc_chain_relu2_gate_f32(const float* gu, int64_t M, int64_t F, float* f);
}

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static float frand() {   /* xorshift, roughly uniform in [-1, 1) */
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (float)((double)(rng_state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main() {
    const int64_t shapes[][3] = {{1, 4, 64}, {3, 20, 192}, {5, 36, 320}, {2, 8, 1088}};
    for (const auto& sh : shapes) {
        const int64_t M = sh[0], N = sh[1], K = sh[2];
        std::vector<float> W((size_t)(N * K));
        for (auto& w : W) w = 0.02f * frand();
        double mean = 0;
        const float beta = orc_absmean_beta(W.data(), N, K, &mean);
        CHECK(beta > 0 && mean > 0);
        std::vector<int8_t> Wt((size_t)(N * K)), Wt2((size_t)(N * K));
        orc_ternarize(W.data(), N, K, beta, Wt.data());
        for (auto t : Wt) CHECK(t >= -1 && t <= 1);
        for (int layout = 0; layout < 2; ++layout) {
            std::vector<uint8_t> packed((size_t)(N * K / 4));
            CHECK(orc_pack(Wt.data(), N, K, layout, packed.data()) == 0);
            CHECK(orc_unpack(packed.data(), N, K, layout, Wt2.data()) == 0);
            CHECK(Wt == Wt2);
        }
        std::vector<float> xf((size_t)(M * K));
        for (auto& x : xf) x = 3.0f * frand();
        std::vector<uint16_t> X((size_t)(M * K));
        orc_f32_to_bf16(xf.data(), M * K, X.data());
        std::vector<int8_t> q((size_t)(M * K));
        std::vector<float> scale((size_t)M);
        std::vector<int32_t> rowsum((size_t)M);
        orc_quant_act(X.data(), M, K, q.data(), scale.data(), rowsum.data());
        for (auto v : q) CHECK(v >= -127);
        std::vector<int32_t> acc((size_t)(M * N));
        orc_matmul_i32(q.data(), Wt.data(), M, N, K, acc.data());
        const int64_t ms[2] = {0, M - 1}, ns[2] = {N - 1, 0};
        int32_t two[2];
        orc_matmul_i32_sampled(q.data(), Wt.data(), N, K, ms, ns, 2, two);
        CHECK(two[0] == acc[(size_t)(0 * N + N - 1)] && two[1] == acc[(size_t)((M - 1) * N)]);
        std::vector<float> y((size_t)(M * N));
        orc_rescale(acc.data(), beta, scale.data(), M, N, y.data());
        std::vector<uint16_t> nb((size_t)(M * K));
        std::vector<double> r64((size_t)M);
        orc_rmsnorm_rows(xf.data(), M, K, nullptr, 1e-5f, nb.data(), r64.data());
        orc_rmsnorm_rows(xf.data(), M, K, xf.data(), 1e-5f, nb.data(), nullptr);
        CHECK(r64[0] > 0);
    }
    {   /* chain glue at a small head geometry: 4 query heads, 1 key/value head of 16 */
        const int64_t M = 3;
        const int n_q = 4, n_kv = 1, hd = 16;
        std::vector<float> qkv((size_t)(M * (n_q + 2 * n_kv) * hd));
        for (auto& v : qkv) v = frand();
        std::vector<uint16_t> a((size_t)(M * n_q * hd));
        std::vector<float> af((size_t)(M * n_q * hd)), h((size_t)(M * n_q * hd));
        orc_chain_attn_stub(qkv.data(), M, n_q, n_kv, hd, a.data());
        orc_chain_attn_f32(qkv.data(), M, n_q, n_kv, hd, af.data());
        orc_chain_residual(af.data(), af.data(), M * n_q * hd, h.data());
        CHECK(h[5] == af[5] + af[5]);
        const int64_t F = 24;
        std::vector<float> gu((size_t)(M * 2 * F)), ff((size_t)(M * F));
        for (auto& v : gu) v = frand();
        std::vector<uint16_t> f((size_t)(M * F));
        orc_chain_relu2_gate(gu.data(), M, F, f.data());
        orc_chain_relu2_gate_f32(gu.data(), M, F, ff.data());
    }
    /* host-only entry points of the library */
    CHECK(bl_packed_bytes(2560, 2560, 1) == 2560 * 2560 / 4);
    CHECK(bl_packed_bytes(6, 64, 0) == 8 * 64 / 4 && bl_packed_bytes(0, 64, 0) == 0);
    CHECK(bl_packed_bytes(2560, 6912, 2) == 2560 * 6960 / 5 && bl_padded_k(65) == 128 && bl_packed_bytes(4, 64, 7) == 0 && bl_packed_bytes(2560, 6912, 3) == 6912 * 2560 / 4);
    CHECK(bl_workspace_bytes(BL_OP_GEMM, 2048, 64, 64) >= 2048 * 4);
    CHECK(bl_status_str(BL_ERR_SHAPE) != nullptr && bl_version() >= 100);
    CHECK(bl_debug_force_path(9) == BL_ERR_VALUE && bl_debug_force_path(0) == BL_OK);
    std::puts("sanitizer run ok");
    return 0;
}
