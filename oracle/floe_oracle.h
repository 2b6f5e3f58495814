/*
 * FloE decode path -- CPU ORACLE (test infrastructure, not a product path).
 *
 * A plain, slow, single-purpose C++17 implementation of what the compressed sparse expert FFN
 * computes, written from the paper's method section.  It exists so that tests can compare the HIP
 * library with something obviously correct; it shares no code, header, table or helper with that
 * library and must never be called from it.  Only the tests, the smoke run and the benchmark's CPU
 * baseline leg may load this library.
 *
 * Precision: every accumulation is done in double, in the index order the formulas state, with no
 * blocking or reordering.  The quantizer is the exception: it works in strict IEEE binary32 (one
 * rounding per operation, no fused multiply-add) because its integer codes must be reproducible
 * bit for bit.
 *
 * Conventions: x is a row vector (Eq. 1).  All matrices are given channel-major: row j holds the d
 * numbers that belong to intermediate channel j (column j of W_up and W_gate, row j of W_down; for
 * W_down this is the transposed storage Sec. 3.4.1 asks for).  Gate and down are co-located per
 * channel as gd[f][2][d] (Sec. 3.4.2, compact layout).  fp16 values travel as uint16_t bit patterns.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against closed forms, brute
 * force, hand-enumerated tiny cases or independent numpy/float64 restatements.  The half-quadratic
 * refinement of (scale, zero) that the paper's quantizer library performs is NOT implemented
 * (the paper gives none of its constants): for that refinement, parity unpinned.
 */
#ifndef FLOE_ORACLE_H
#define FLOE_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* number of worker threads used by the embarrassingly parallel outer loops (default 1). */
void floe_oracle_set_threads(int n);
int floe_oracle_get_threads(void);

/* fp16 helpers exposed for the tests (exact widening; round-to-nearest-even narrowing). */
float floe_oracle_half_to_float(uint16_t h);
uint16_t floe_oracle_float_to_half(float x);
uint16_t floe_oracle_double_to_half(double x);

/* number of 32-bit words that hold one channel's d codes of `bits` bits. */
int floe_oracle_words_per_channel(int d, int bits);

/*
 * Sec. 3.2.2 (quantized up projection), asymmetric uniform group quantizer:
 * for channel j and group G of `group` consecutive reduction indices i,
 *   mn, mx = min / max of the group;  scale = fp16((mx - mn) / qmax),  qmax = 2^bits - 1
 *   zero = fp16(-mn / scale);  q = clamp(rint(w / scale + zero), 0, qmax)
 * (scale and zero are rounded to fp16 first and the rounded values are used for q).
 * Degenerate group (mx == mn, or scale below the smallest normal fp16): scale = 1, zero = fp16(-mn), q = 0.
 * Codes of a channel form a little-endian bit stream: code i sits at bits [bits*i, bits*i+bits)
 * of the channel's words.  Returns 0, or -1 for an invalid shape.
 */
int floe_oracle_quantize(const uint16_t* w_cm, int f, int d, int bits, int group,
                         uint32_t* codes, uint16_t* scale, uint16_t* zero);

/* w_hat[j][i] = (q - zero) * scale, evaluated in binary32 and not re-rounded to fp16. */
int floe_oracle_dequantize(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                           int f, int d, int bits, int group, float* w_hat);

/* Alg. 1 line 2 with the quantized matrix: v_j = sum_i x_i * w_hat[j][i] (double sum, i ascending),
 * stored as float. */
int floe_oracle_up_gemv(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                        int f, int d, int bits, int group, const uint16_t* x, float* v);

/* Alg. 1 line 3: ascending list of j with |v_j| > tau (strict).  Returns K. */
int floe_oracle_select(const float* v, int f, float tau, int32_t* idx);

/* Eq. 6 applied to one token's |v|: the smallest t with F(t) >= pct/100 where F is the empirical CDF
 * of |v_j|, i.e. the z-th smallest |v_j| with z = ceil(f*pct/100); z = 0 gives -1 (keep everything). */
float floe_oracle_threshold_for_sparsity(const float* v, int f, int pct);

/* Alg. 1 lines 4-5 on a given index list.  gd is [rows][2][d]; when `staged` is 0 row idx[k] is used,
 * when 1 row k holds channel idx[k].  h (K doubles, may be NULL) receives SiLU(x.W_gate[:,j]) * v_j;
 * y (d doubles) receives sum_k h_k * W_down[j_k, :]. */
int floe_oracle_sparse_ffn(const uint16_t* gd, int staged, int d, const uint16_t* x, const float* v,
                           const int32_t* idx, int K, double* h, double* y);

/* Eq. 1, the dense SwiGLU expert, with an arbitrary float up matrix w_up[f][d] (channel-major). */
int floe_oracle_dense_ffn(const float* w_up, const uint16_t* gd, int d, int f, const uint16_t* x, double* y);

/* The sparse expert forward a^S(x) of Sec. 3.2.1 (Eq. 1 with S_t of Eq. 5 applied to x.W_up) evaluated
 * literally: dense loops over all f channels, strict comparison as in Alg. 1, no index list. */
int floe_oracle_masked_dense_ffn(const float* w_up, const uint16_t* gd, int d, int f, const uint16_t* x,
                                 float tau, double* y);

/*
 * The three candidates for sparsification of Sec. 3.2.1 (Eq. 3-5): S_t applied to
 *   which = 0: a_up = x.W_up          (what FloE uses; equals floe_oracle_masked_dense_ffn on the same a_up),
 *   which = 1: a_gate = SiLU(x.W_gate),
 *   which = 2: a_down = a_gate * a_up,
 * inside the expert forward of Eq. 1: y = sum over the kept channels of a_gate_j * a_up_j * W_down[j, :].
 * a_up is given (the caller computes it, e.g. with floe_oracle_up_gemv); the comparison |a| > tau is strict and taken
 * on the binary32 value of a.  Optional outputs: idx / K_out (kept channels, ascending), act (the f values compared).
 */
int floe_oracle_sparsified_ffn(int which, const uint16_t* gd, int d, int f, const uint16_t* x, const float* a_up,
                               float tau, double* y, int32_t* idx, int32_t* K_out, double* act);

/* Router: logits_e = x . W_r[e], softmax (max-subtracted), top_k by probability (ties -> lower id),
 * weights p_e / sum_selected(p) if renormalize else p_e.  ids are listed by descending probability. */
int floe_oracle_router(const uint16_t* router_cm, int n_experts, int d, const uint16_t* x,
                       int top_k, int renormalize, int32_t* ids, double* weights, double* probs);

typedef struct {
    const uint32_t* codes;
    const uint16_t* scale;
    const uint16_t* zero;
    const uint16_t* gd; /* [f][2][d] */
} floe_oracle_expert;

/*
 * One MoE layer at decode for T independent tokens: route, run the sparse FFN of every selected
 * expert (and of the n_shared always-on experts that follow the routed ones in `experts`, weight 1),
 * combine with the router weights in double, round once to fp16.
 * tau is [T][n_experts + n_shared] (only the entries of the experts a token uses are read).
 * Optional outputs (may be NULL): ids [T][top_k], weights [T][top_k],
 * counts [T][top_k + n_shared] = K of each (token, slot), y_f64 [T][d] = the unrounded output.
 */
int floe_oracle_moe_layer(const floe_oracle_expert* experts, int n_experts, int n_shared, int top_k,
                          int renormalize, const uint16_t* router_cm, int d, int f, int bits, int group,
                          const uint16_t* x, int T, const float* tau, uint16_t* out,
                          int32_t* ids, double* weights, int32_t* counts, double* y_f64);

/* Sec. 3.4.2: rows idx[0..K) of a compact [f][2][d] matrix copied to dst[k][2][d]. */
int floe_oracle_stage_rows(const uint16_t* gd, int d, const int32_t* idx, int K, uint16_t* dst);

#ifdef __cplusplus
}
#endif
#endif
