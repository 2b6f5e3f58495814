// Runs every entry point of the CPU oracle on small, awkward inputs (ragged sizes, empty lists, degenerate groups,
// every bit width, several threads).  Built by tests/test_oracle_sanitizers.py with -fsanitize=address,undefined and
// -fno-sanitize-recover: any out-of-bounds access, use of uninitialised heap, signed overflow or misaligned access in
// the oracle ends the run with a report and a non-zero status.  The values themselves are pinned by test_oracle_*.py.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../oracle/floe_oracle.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform() {
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static uint16_t half_of(double x) { return floe_oracle_double_to_half(x); }
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int run_shape(int d, int f, int bits, int group, int T, int threads) {
    floe_oracle_set_threads(threads);
    const int wpc = floe_oracle_words_per_channel(d, bits), G = d / group;
    std::vector<uint16_t> w((size_t)f * d), gd((size_t)f * 2 * d), x((size_t)T * d);
    for (auto& v : w) v = half_of((uniform() - 0.5) * 0.08);
    for (auto& v : gd) v = half_of((uniform() - 0.5) * 0.08);
    for (auto& v : x) v = half_of((uniform() - 0.5) * 4.0);
    for (int i = 0; i < group && f > 1; ++i) w[(size_t)d + i] = half_of(0.25);  // a degenerate group in channel 1
    std::vector<uint32_t> codes((size_t)f * wpc);
    std::vector<uint16_t> scale((size_t)f * G), zero((size_t)f * G);
    CHECK(floe_oracle_quantize(w.data(), f, d, bits, group, codes.data(), scale.data(), zero.data()) == 0);
    std::vector<float> w_hat((size_t)f * d), v(f);
    CHECK(floe_oracle_dequantize(codes.data(), scale.data(), zero.data(), f, d, bits, group, w_hat.data()) == 0);
    CHECK(floe_oracle_up_gemv(codes.data(), scale.data(), zero.data(), f, d, bits, group, x.data(), v.data()) == 0);
    std::vector<int32_t> idx(f);
    std::vector<double> y(d), h(f), act(f);
    const int pcts[4] = {0, 50, 90, 100};
    for (int pct : pcts) {
        const float tau = floe_oracle_threshold_for_sparsity(v.data(), f, pct);
        const int K = floe_oracle_select(v.data(), f, tau, idx.data());
        CHECK(K >= 0 && K <= f);
        CHECK(floe_oracle_sparse_ffn(gd.data(), 0, d, x.data(), v.data(), idx.data(), K, K ? h.data() : nullptr, y.data()) == 0);
        std::vector<uint16_t> staged((size_t)(K ? K : 1) * 2 * d);
        CHECK(floe_oracle_stage_rows(gd.data(), d, idx.data(), K, staged.data()) == 0);
        CHECK(floe_oracle_sparse_ffn(staged.data(), 1, d, x.data(), v.data(), idx.data(), K, nullptr, y.data()) == 0);
        CHECK(floe_oracle_masked_dense_ffn(w_hat.data(), gd.data(), d, f, x.data(), tau, y.data()) == 0);
        for (int which = 0; which < 3; ++which) {
            int32_t Kout = -1;
            CHECK(floe_oracle_sparsified_ffn(which, gd.data(), d, f, x.data(), v.data(), tau, y.data(), idx.data(), &Kout,
                                             act.data()) == 0);
            CHECK(Kout >= 0 && Kout <= f);
        }
    }
    CHECK(floe_oracle_dense_ffn(w_hat.data(), gd.data(), d, f, x.data(), y.data()) == 0);
    // a layer of three such experts (two routed, one shared)
    const int n = 2, n_shared = 1, top_k = 2;
    std::vector<uint16_t> router((size_t)n * d);
    for (auto& r : router) r = half_of((uniform() - 0.5) * 0.08);
    std::vector<int32_t> ids(top_k);
    std::vector<double> wts(top_k), probs(n);
    CHECK(floe_oracle_router(router.data(), n, d, x.data(), top_k, 1, ids.data(), wts.data(), probs.data()) == 0);
    floe_oracle_expert ex[3];
    for (auto& e : ex) e = floe_oracle_expert{codes.data(), scale.data(), zero.data(), gd.data()};
    std::vector<float> tau((size_t)T * (n + n_shared), 0.5f);
    std::vector<uint16_t> out((size_t)T * d);
    std::vector<int32_t> lids((size_t)T * top_k), counts((size_t)T * (top_k + n_shared));
    std::vector<double> lw((size_t)T * top_k), yf((size_t)T * d);
    CHECK(floe_oracle_moe_layer(ex, n, n_shared, top_k, 0, router.data(), d, f, bits, group, x.data(), T, tau.data(), out.data(),
                                lids.data(), lw.data(), counts.data(), yf.data()) == 0);
    CHECK(floe_oracle_moe_layer(ex, n, n_shared, top_k, 1, router.data(), d, f, bits, group, x.data(), T, tau.data(), out.data(),
                                nullptr, nullptr, nullptr, nullptr) == 0);
    return 0;
}

int main() {
    for (int h = 0; h < 65536; h += 257) (void)floe_oracle_float_to_half(floe_oracle_half_to_float((uint16_t)h));
    const int bits_all[5] = {1, 2, 3, 4, 8};
    for (int bits : bits_all) {
        if (run_shape(64, 1, bits, 32, 1, 1)) return 1;      // one channel
        if (run_shape(128, 7, bits, 64, 2, 3)) return 1;     // ragged, more threads than some loops have items
        if (run_shape(256, 33, bits, 128, 3, 2)) return 1;
    }
    // invalid shapes are refused, not read
    std::vector<uint16_t> w(64);
    std::vector<uint32_t> c(64);
    std::vector<uint16_t> s(64), z(64);
    if (floe_oracle_quantize(w.data(), 1, 60, 2, 64, c.data(), s.data(), z.data()) == 0) return 1;  // d % group != 0
    if (floe_oracle_quantize(w.data(), 1, 64, 5, 64, c.data(), s.data(), z.data()) == 0) return 1;  // width not offered
    std::puts("oracle sanitizer run: ok");
    return 0;
}
