// FloE decode path -- CPU ORACLE (test infrastructure; see floe_oracle.h for the contract).
//
// Every function follows the paper's formulas in their stated order with double accumulation.
// Nothing here is blocked, fused, vectorised by hand or shared with the HIP library.
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC (see oracle/build.py).
#include "floe_oracle.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <thread>
#include <vector>

namespace {

int g_threads = 1;

// Runs body(j) for j in [0, n) on g_threads workers; iterations are independent and each writes
// only its own outputs, so the result does not depend on the thread count.
void parallel_for(int n, const std::function<void(int)>& body) {
    int nt = std::max(1, std::min(g_threads, n));
    if (nt == 1) {
        for (int j = 0; j < n; ++j) body(j);
        return;
    }
    std::vector<std::thread> pool;
    for (int t = 0; t < nt; ++t) {
        pool.emplace_back([=, &body]() {
            int lo = (int)((long long)n * t / nt), hi = (int)((long long)n * (t + 1) / nt);
            for (int j = lo; j < hi; ++j) body(j);
        });
    }
    for (auto& th : pool) th.join();
}

// ---- IEEE binary16 <-> binary32/64, written out on the bit level -------------------------------

float half_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    int e = (h >> 10) & 0x1F;
    uint32_t m = h & 0x3FF;
    if (e == 0) {                       // zero or subnormal: m * 2^-24
        float mag = std::ldexp((float)m, -24);
        return sign ? -mag : mag;
    }
    uint32_t bits;
    if (e == 31) bits = sign | 0x7F800000u | (m << 13);            // inf / nan
    else bits = sign | ((uint32_t)(e - 15 + 127) << 23) | (m << 13);
    float f;
    std::memcpy(&f, &bits, 4);
    return f;
}

// Round a finite double to the nearest binary16 (ties to even); overflow gives infinity.
uint16_t double_to_half(double x) {
    uint16_t sign = std::signbit(x) ? 0x8000 : 0;
    if (std::isnan(x)) return sign | 0x7E00;
    double a = std::fabs(x);
    if (std::isinf(a)) return sign | 0x7C00;
    if (a == 0.0) return sign;
    int e;
    std::frexp(a, &e);                  // a = m * 2^e, m in [0.5, 1)  ->  a in [2^(e-1), 2^e)
    int exp = e - 1;                    // unbiased exponent of the leading bit
    if (exp < -14) exp = -14;           // subnormal range shares the spacing 2^-24
    double ulp = std::ldexp(1.0, exp - 10);
    double q = a / ulp;                 // exact: a power-of-two scaling
    double r = std::nearbyint(q);       // default rounding mode is to-nearest-even
    double v = r * ulp;
    if (v >= 65520.0) return sign | 0x7C00;
    // re-derive exponent/mantissa from the rounded value (rounding may carry into the next binade)
    if (v < std::ldexp(1.0, -14)) return sign | (uint16_t)std::lround(v / std::ldexp(1.0, -24));
    int e2;
    std::frexp(v, &e2);
    int ex = e2 - 1;
    double frac = v / std::ldexp(1.0, ex) - 1.0;       // [0, 1)
    uint16_t mant = (uint16_t)std::lround(frac * 1024.0);
    return sign | (uint16_t)((ex + 15) << 10) | mant;
}

// binary32 -> binary16 is a single rounding of an exactly representable double.
uint16_t float_to_half(float x) { return double_to_half((double)x); }

bool shape_ok(int f, int d, int bits, int group) {
    if (f < 0 || d <= 0 || group <= 0) return false;
    // the widths of the paper's sensitivity study (Sec. 3.2.2: INT8, INT4, INT3, INT2, INT1); the arithmetic is the same
    if (bits != 1 && bits != 2 && bits != 3 && bits != 4 && bits != 8) return false;
    if (d % group != 0) return false;
    if ((group * bits) % 32 != 0) return false;
    return true;
}

inline uint32_t get_code(const uint32_t* words, int i, int bits) {
    long long bit = (long long)i * bits;
    int w = (int)(bit >> 5), o = (int)(bit & 31);
    uint64_t two = words[w];
    if (o + bits > 32) two |= (uint64_t)words[w + 1] << 32;
    return (uint32_t)((two >> o) & ((1u << bits) - 1));
}

inline void put_code(uint32_t* words, int i, int bits, uint32_t q) {
    long long bit = (long long)i * bits;
    int w = (int)(bit >> 5), o = (int)(bit & 31);
    words[w] |= q << o;
    if (o + bits > 32) words[w + 1] |= q >> (32 - o);
}

inline float dequant_one(uint32_t q, uint16_t zero_h, uint16_t scale_h) {
    volatile float diff = (float)q - half_to_float(zero_h);   // one rounding
    return diff * half_to_float(scale_h);                      // one rounding
}

inline double silu(double g) { return g / (1.0 + std::exp(-g)); }   // Eq. 2

}  // namespace

extern "C" {

void floe_oracle_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int floe_oracle_get_threads(void) { return g_threads; }

float floe_oracle_half_to_float(uint16_t h) { return half_to_float(h); }
uint16_t floe_oracle_float_to_half(float x) { return float_to_half(x); }
uint16_t floe_oracle_double_to_half(double x) { return double_to_half(x); }

int floe_oracle_words_per_channel(int d, int bits) { return (int)(((long long)d * bits + 31) / 32); }

int floe_oracle_quantize(const uint16_t* w_cm, int f, int d, int bits, int group,
                         uint32_t* codes, uint16_t* scale, uint16_t* zero) {
    if (!shape_ok(f, d, bits, group)) return -1;
    const int wpc = floe_oracle_words_per_channel(d, bits);
    const int G = d / group;
    const float qmax = (float)((1 << bits) - 1);
    parallel_for(f, [&](int j) {
        const uint16_t* w = w_cm + (size_t)j * d;
        uint32_t* cw = codes + (size_t)j * wpc;
        std::memset(cw, 0, sizeof(uint32_t) * wpc);
        for (int gi = 0; gi < G; ++gi) {
            float mn = half_to_float(w[gi * group]), mx = mn;
            for (int i = 1; i < group; ++i) {
                float a = half_to_float(w[gi * group + i]);
                mn = std::min(mn, a);
                mx = std::max(mx, a);
            }
            volatile float range = mx - mn;
            volatile float s32 = range / qmax;
            uint16_t sh = float_to_half(s32);
            float S = half_to_float(sh);
            bool degenerate = !(mx > mn) || !(S >= 6.103515625e-05f) || std::isinf(S);
            uint16_t zh;
            if (degenerate) {
                sh = 0x3C00;  // 1.0
                zh = float_to_half(-mn);
                // all codes stay 0: w_hat = (0 - zero) * 1 = mn
            } else {
                volatile float z32 = (-mn) / S;
                float zc = std::min(std::max((float)z32, -65504.0f), 65504.0f);
                zh = float_to_half(zc);
                float Z = half_to_float(zh);
                for (int i = 0; i < group; ++i) {
                    float a = half_to_float(w[gi * group + i]);
                    volatile float t = a / S;          // correctly rounded binary32 division
                    volatile float u = t + Z;          // separate rounding (no fused multiply-add)
                    float r = std::nearbyintf(u);      // ties to even
                    r = std::min(std::max(r, 0.0f), qmax);
                    put_code(cw, gi * group + i, bits, (uint32_t)r);
                }
            }
            scale[(size_t)j * G + gi] = sh;
            zero[(size_t)j * G + gi] = zh;
        }
    });
    return 0;
}

int floe_oracle_dequantize(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                           int f, int d, int bits, int group, float* w_hat) {
    if (!shape_ok(f, d, bits, group)) return -1;
    const int wpc = floe_oracle_words_per_channel(d, bits);
    const int G = d / group;
    parallel_for(f, [&](int j) {
        for (int i = 0; i < d; ++i) {
            uint32_t q = get_code(codes + (size_t)j * wpc, i, bits);
            size_t m = (size_t)j * G + i / group;
            w_hat[(size_t)j * d + i] = dequant_one(q, zero[m], scale[m]);
        }
    });
    return 0;
}

int floe_oracle_up_gemv(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                        int f, int d, int bits, int group, const uint16_t* x, float* v) {
    if (!shape_ok(f, d, bits, group)) return -1;
    const int wpc = floe_oracle_words_per_channel(d, bits);
    const int G = d / group;
    parallel_for(f, [&](int j) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i) {
            uint32_t q = get_code(codes + (size_t)j * wpc, i, bits);
            size_t m = (size_t)j * G + i / group;
            acc += (double)half_to_float(x[i]) * (double)dequant_one(q, zero[m], scale[m]);
        }
        v[j] = (float)acc;
    });
    return 0;
}

int floe_oracle_select(const float* v, int f, float tau, int32_t* idx) {
    int K = 0;
    for (int j = 0; j < f; ++j)
        if (std::fabs(v[j]) > tau) idx[K++] = j;
    return K;
}

float floe_oracle_threshold_for_sparsity(const float* v, int f, int pct) {
    long long z = ((long long)f * pct + 99) / 100;   // ceil(f * pct / 100)
    if (z <= 0) return -1.0f;
    if (z > f) z = f;
    std::vector<float> a(f);
    for (int j = 0; j < f; ++j) a[j] = std::fabs(v[j]);
    std::sort(a.begin(), a.end());
    return a[z - 1];
}

int floe_oracle_sparse_ffn(const uint16_t* gd, int staged, int d, const uint16_t* x, const float* v,
                           const int32_t* idx, int K, double* h, double* y) {
    if (d <= 0 || K < 0) return -1;
    std::vector<double> hh(K);
    parallel_for(K, [&](int k) {
        int j = idx[k];
        const uint16_t* gate = gd + (size_t)(staged ? k : j) * 2 * d;
        double g = 0.0;
        for (int i = 0; i < d; ++i) g += (double)half_to_float(x[i]) * (double)half_to_float(gate[i]);
        hh[k] = silu(g) * (double)v[j];              // Alg. 1 line 4
    });
    if (h) std::copy(hh.begin(), hh.end(), h);
    parallel_for(d, [&](int i) {
        double acc = 0.0;
        for (int k = 0; k < K; ++k) {                // Alg. 1 line 5
            const uint16_t* down = gd + (size_t)(staged ? k : idx[k]) * 2 * d + d;
            acc += hh[k] * (double)half_to_float(down[i]);
        }
        y[i] = acc;
    });
    return 0;
}

int floe_oracle_dense_ffn(const float* w_up, const uint16_t* gd, int d, int f, const uint16_t* x, double* y) {
    if (d <= 0 || f < 0) return -1;
    std::vector<double> a_down(f);
    parallel_for(f, [&](int j) {
        double g = 0.0, u = 0.0;
        const uint16_t* gate = gd + (size_t)j * 2 * d;
        for (int i = 0; i < d; ++i) {
            double xi = (double)half_to_float(x[i]);
            g += xi * (double)half_to_float(gate[i]);
            u += xi * (double)w_up[(size_t)j * d + i];
        }
        a_down[j] = silu(g) * u;                     // Eq. 1 / Eq. 4
    });
    parallel_for(d, [&](int i) {
        double acc = 0.0;
        for (int j = 0; j < f; ++j) acc += a_down[j] * (double)half_to_float(gd[(size_t)j * 2 * d + d + i]);
        y[i] = acc;
    });
    return 0;
}

int floe_oracle_masked_dense_ffn(const float* w_up, const uint16_t* gd, int d, int f, const uint16_t* x,
                                 float tau, double* y) {
    if (d <= 0 || f < 0) return -1;
    std::vector<double> a_down(f);
    parallel_for(f, [&](int j) {
        double g = 0.0, u = 0.0;
        const uint16_t* gate = gd + (size_t)j * 2 * d;
        for (int i = 0; i < d; ++i) {
            double xi = (double)half_to_float(x[i]);
            g += xi * (double)half_to_float(gate[i]);
            u += xi * (double)w_up[(size_t)j * d + i];
        }
        float uf = (float)u;                                    // v is carried as binary32
        double s = (std::fabs(uf) > tau) ? (double)uf : 0.0;    // S_t, strict as in Alg. 1
        a_down[j] = silu(g) * s;
    });
    parallel_for(d, [&](int i) {
        double acc = 0.0;
        for (int j = 0; j < f; ++j) acc += a_down[j] * (double)half_to_float(gd[(size_t)j * 2 * d + d + i]);
        y[i] = acc;
    });
    return 0;
}

int floe_oracle_sparsified_ffn(int which, const uint16_t* gd, int d, int f, const uint16_t* x, const float* a_up,
                               float tau, double* y, int32_t* idx, int32_t* K_out, double* act) {
    if (d <= 0 || f < 0 || which < 0 || which > 2) return -1;
    // Eq. 3-4: the three activations, every channel, dense loops
    std::vector<double> a_gate(f), a_down(f);
    parallel_for(f, [&](int j) {
        double g = 0.0;
        const uint16_t* gate = gd + (size_t)j * 2 * d;
        for (int i = 0; i < d; ++i) g += (double)half_to_float(x[i]) * (double)half_to_float(gate[i]);
        a_gate[j] = silu(g);
        a_down[j] = a_gate[j] * (double)a_up[j];
    });
    // Eq. 5 on the chosen activation, compared as binary32 and strictly (as Alg. 1 does for a_up)
    std::vector<char> keep(f);
    int K = 0;
    for (int j = 0; j < f; ++j) {
        const double a = which == 0 ? (double)a_up[j] : (which == 1 ? a_gate[j] : a_down[j]);
        if (act) act[j] = a;
        keep[j] = std::fabs((float)a) > tau;
        if (keep[j]) {
            if (idx) idx[K] = j;
            ++K;
        }
    }
    if (K_out) *K_out = K;
    // Eq. 1 with the sparsified activation in place: a channel that was dropped contributes exactly nothing
    parallel_for(d, [&](int i) {
        double acc = 0.0;
        for (int j = 0; j < f; ++j)
            if (keep[j]) acc += a_down[j] * (double)half_to_float(gd[(size_t)j * 2 * d + d + i]);
        y[i] = acc;
    });
    return 0;
}

int floe_oracle_router(const uint16_t* router_cm, int n_experts, int d, const uint16_t* x,
                       int top_k, int renormalize, int32_t* ids, double* weights, double* probs) {
    if (n_experts <= 0 || top_k < 0 || top_k > n_experts || d <= 0) return -1;
    std::vector<double> p(n_experts);
    double mx = -INFINITY;
    for (int e = 0; e < n_experts; ++e) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i)
            acc += (double)half_to_float(x[i]) * (double)half_to_float(router_cm[(size_t)e * d + i]);
        p[e] = acc;
        mx = std::max(mx, acc);
    }
    double sum = 0.0;
    for (int e = 0; e < n_experts; ++e) { p[e] = std::exp(p[e] - mx); sum += p[e]; }
    for (int e = 0; e < n_experts; ++e) p[e] /= sum;
    if (probs) std::copy(p.begin(), p.end(), probs);
    std::vector<char> taken(n_experts, 0);
    double sel = 0.0;
    for (int r = 0; r < top_k; ++r) {
        int best = -1;
        for (int e = 0; e < n_experts; ++e)
            if (!taken[e] && (best < 0 || p[e] > p[best])) best = e;   // ties keep the lower id
        taken[best] = 1;
        ids[r] = best;
        weights[r] = p[best];
        sel += p[best];
    }
    if (renormalize)
        for (int r = 0; r < top_k; ++r) weights[r] /= sel;
    return 0;
}

int floe_oracle_moe_layer(const floe_oracle_expert* experts, int n_experts, int n_shared, int top_k,
                          int renormalize, const uint16_t* router_cm, int d, int f, int bits, int group,
                          const uint16_t* x, int T, const float* tau, uint16_t* out,
                          int32_t* ids, double* weights, int32_t* counts, double* y_f64) {
    if (!shape_ok(f, d, bits, group) || T < 0 || n_shared < 0) return -1;
    const int slots = top_k + n_shared;
    const int n_all = n_experts + n_shared;
    std::vector<float> v(f);
    std::vector<int32_t> idx(f);
    std::vector<double> y(d), acc(d);
    std::vector<int32_t> sel(std::max(1, top_k));
    std::vector<double> w(std::max(1, top_k));
    for (int t = 0; t < T; ++t) {
        const uint16_t* xt = x + (size_t)t * d;
        if (top_k > 0) {
            int rc = floe_oracle_router(router_cm, n_experts, d, xt, top_k, renormalize, sel.data(), w.data(), nullptr);
            if (rc) return rc;
        }
        std::fill(acc.begin(), acc.end(), 0.0);
        for (int s = 0; s < slots; ++s) {
            int e = s < top_k ? sel[s] : n_experts + (s - top_k);
            double we = s < top_k ? w[s] : 1.0;
            const floe_oracle_expert& ex = experts[e];
            floe_oracle_up_gemv(ex.codes, ex.scale, ex.zero, f, d, bits, group, xt, v.data());
            int K = floe_oracle_select(v.data(), f, tau[(size_t)t * n_all + e], idx.data());
            floe_oracle_sparse_ffn(ex.gd, 0, d, xt, v.data(), idx.data(), K, nullptr, y.data());
            for (int i = 0; i < d; ++i) acc[i] += we * y[i];
            if (counts) counts[(size_t)t * slots + s] = K;
            if (s < top_k) {
                if (ids) ids[(size_t)t * top_k + s] = e;
                if (weights) weights[(size_t)t * top_k + s] = we;
            }
        }
        for (int i = 0; i < d; ++i) {
            out[(size_t)t * d + i] = double_to_half(acc[i]);
            if (y_f64) y_f64[(size_t)t * d + i] = acc[i];
        }
    }
    return 0;
}

int floe_oracle_stage_rows(const uint16_t* gd, int d, const int32_t* idx, int K, uint16_t* dst) {
    if (d <= 0 || K < 0) return -1;
    for (int k = 0; k < K; ++k)
        std::memcpy(dst + (size_t)k * 2 * d, gd + (size_t)idx[k] * 2 * d, sizeof(uint16_t) * 2 * d);
    return 0;
}

}  // extern "C"
