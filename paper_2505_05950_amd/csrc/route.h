// Softmax + top-k of the router (S1), shared by the stand-alone router kernel and by the GEMV kernel
// that routes in place.  Run by ONE thread on logits held in LDS; n_experts is small (<= 1024).
#pragma once

#include "floe_dev.h"

namespace floe {

// prob[0..n) holds the logits on entry and is destroyed.  sel_id / sel_w receive the top_k experts by
// descending probability (ties keep the lower id) with weight p_e, or p_e / sum of the selected p when
// renormalize is set.  The n_shared always-on experts follow with ids n, n+1, ... and weight 1.
__device__ __forceinline__ void route_select(float* prob, int n, int top_k, int n_shared, int renormalize, int* sel_id,
                                             float* sel_w) {
    if (top_k > 0) {
        float mx = prob[0];
        for (int e = 1; e < n; ++e) mx = fmaxf(mx, prob[e]);
        float sum = 0.0f;
        for (int e = 0; e < n; ++e) {
            const float p = expf(prob[e] - mx);
            prob[e] = p;
            sum += p;
        }
        float sel = 0.0f;
        for (int r = 0; r < top_k; ++r) {
            int best = -1;
            float bp = -1.0f;
            for (int e = 0; e < n; ++e) {
                const float p = prob[e];
                if (p > bp) { bp = p; best = e; }  // strict: ties keep the lower id
            }
            if (best < 0) best = 0;  // only reachable with NaN logits: stay in bounds
            prob[best] = -2.0f;      // taken
            const float pw = bp / sum;
            sel_id[r] = best;
            sel_w[r] = pw;
            sel += pw;
        }
        if (renormalize)
            for (int r = 0; r < top_k; ++r) sel_w[r] /= sel;
    }
    for (int s = 0; s < n_shared; ++s) {
        sel_id[top_k + s] = n + s;
        sel_w[top_k + s] = 1.0f;
    }
}

// The same selection for n <= 16 experts, done by the first 16 lanes of one wave with the logits in
// registers (no serial LDS round trips).  Every lane of the wave must call it; `logit` is the lane's
// own logit for lane < n (ignored otherwise).  Bit-identical to route_select: same expf, same
// left-to-right sums, same tie rule.  Split in two so that a caller can act on the expert ids (start
// loading weights) before the divisions that give the routing weights.
struct Pick16 {
    float p;    // lane r (< top_k) of every row of 16: unnormalised probability of the r-th pick
    int id;     // lane r: its expert id
    float sum;  // softmax denominator (all lanes)
};
__device__ __forceinline__ Pick16 route_pick_wave16(float logit, int lane, int n, int top_k) {
    const int l16 = lane & 15;
    const bool live = l16 < n;
    const float mx = row16_allreduce_max(live ? logit : -INFINITY);
    const float p = live ? expf(logit - mx) : 0.0f;
    Pick16 out;
    // sum in ascending expert order, exactly like the serial loop (lane e of row 0 holds p_e)
    out.sum = 0.0f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const float pe = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, p), e));
        if (e < n) out.sum += pe;
    }
    float cur = live ? p : -3.0f;
    out.p = 0.0f;
    out.id = 0;
    for (int r = 0; r < top_k; ++r) {
        // arg-max with ties to the lower id: (value, id) pairs rotate around the row of 16
        float bv = cur;
        int bi = l16;
#define FLOE_ARGMAX_STEP(CTRL)                                               \
    {                                                                        \
        const float ov = dpp_movf<CTRL>(bv);                                 \
        const int oi = dpp_movi<CTRL>(bi);                                   \
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }          \
    }
        FLOE_ARGMAX_STEP(0x128) FLOE_ARGMAX_STEP(0x124) FLOE_ARGMAX_STEP(0x122) FLOE_ARGMAX_STEP(0x121)
#undef FLOE_ARGMAX_STEP
        if (l16 == r) { out.p = bv; out.id = bi; }
        if (l16 == bi) cur = -2.0f;  // taken
    }
    return out;
}
// The pick for n <= 64 experts (lane e of the wave holds expert e), result laid out like route_pick_wave16's: lane r
// (< top_k <= 16) receives the r-th pick.  The sum of the exponentials is a DPP tree, as in the stand-alone router's
// wave-wide selection, so both give the same bits.
__device__ __forceinline__ Pick16 route_pick_wave64(float logit, int lane, int n, int top_k) {
    const bool live = lane < n;
    auto lane_value = [](float v, int l) {
        return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
    };
    float mx = row16_allreduce_max(live ? logit : -INFINITY);
    mx = fmaxf(fmaxf(lane_value(mx, 0), lane_value(mx, 16)), fmaxf(lane_value(mx, 32), lane_value(mx, 48)));
    const float p = live ? expf(logit - mx) : 0.0f;
    Pick16 out;
    out.sum = wave_allreduce_sum(p);
    out.p = 0.0f;
    out.id = 0;
    float cur = live ? p : -3.0f;
    for (int r = 0; r < top_k; ++r) {
        // arg-max with ties to the lower id: inside each row of 16 on the DPP path, then the four row winners (in
        // ascending id order, so a strict comparison keeps the lower id) through scalar registers
        float bv = cur;
        int bi = lane;
#define FLOE_ARGMAX_STEP(CTRL)                                               \
    {                                                                        \
        const float ov = dpp_movf<CTRL>(bv);                                 \
        const int oi = dpp_movi<CTRL>(bi);                                   \
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }          \
    }
        FLOE_ARGMAX_STEP(0x128) FLOE_ARGMAX_STEP(0x124) FLOE_ARGMAX_STEP(0x122) FLOE_ARGMAX_STEP(0x121)
#undef FLOE_ARGMAX_STEP
        float wv = lane_value(bv, 0);
        int wi = __builtin_amdgcn_readlane(bi, 0);
#pragma unroll
        for (int row = 1; row < 4; ++row) {
            const float ov = lane_value(bv, 16 * row);
            const int oi = __builtin_amdgcn_readlane(bi, 16 * row);
            if (ov > wv) { wv = ov; wi = oi; }
        }
        if (lane == r) { out.p = wv; out.id = wi; }
        if (lane == wi) cur = -2.0f;  // taken
    }
    return out;
}
// routing weight of the lane's pick (lane < top_k): p / sum, or that over the sum of the picked ones
__device__ __forceinline__ float route_weight_wave16(const Pick16& pk, int top_k, int renormalize) {
    const float pw = pk.p / pk.sum;
    float sel = 0.0f;
    for (int r = 0; r < top_k; ++r)
        sel += __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pw), r));
    return renormalize ? pw / sel : pw;
}
__device__ __forceinline__ void route_select_wave16(float logit, int lane, int n, int top_k, int n_shared,
                                                    int renormalize, int* sel_id, float* sel_w) {
    if (top_k > 0) {
        const Pick16 pk = route_pick_wave16(logit, lane, n, top_k);
        const float w = route_weight_wave16(pk, top_k, renormalize);
        if (lane < top_k) {
            sel_id[lane] = pk.id;
            sel_w[lane] = w;
        }
    }
    if (lane < n_shared) {
        sel_id[top_k + lane] = n + lane;
        sel_w[top_k + lane] = 1.0f;
    }
}

// What a kernel that routes in place needs (layer path).
struct RouteArgs {
    const h16* router_cm;     // [n_experts][d]
    const float* logits;      // nullptr: the kernel forms x . W_r itself (n_experts <= 16); else [T][n_experts], computed
                              // by a kernel in front (n_experts <= 64)
    const float* tau;         // threshold of (token t, expert e) at tau[t * tau_stride_t + e]
    int32_t tau_stride_t;
    int32_t n_experts, top_k, n_shared, renormalize;
    const DevExpert* table;   // all experts of the layer
    DevExpert* task_table;    // [n_tasks] out (written by the first workgroup of each task)
    int32_t* task_expert;     // [n_tasks] out
    float* task_weight;       // [n_tasks] out
    float* task_tau;          // [n_tasks] out
};

// Router logits of one token by a workgroup of NW waves, for kernels that route in place: a wave per piece of an
// expert's row (kParts pieces per row), two pieces in flight per wave, fully coalesced 16-byte loads.
// plog[e * kParts + part] receives the partial dot product; the caller sums the parts after a barrier.
template <int D, int NW, int kParts>
__device__ __forceinline__ void route_logits_to_lds(const h16* __restrict__ xt, const RouteArgs& ro, int wave, int lane,
                                                    float* plog) {
    constexpr int NVR = D / 512 / kParts;
    const int n_items = ro.n_experts * kParts;
    const uint4* xp4 = reinterpret_cast<const uint4*>(xt);
    for (int it0 = wave; it0 < n_items; it0 += 2 * NW) {
        uint4 w[2][NVR], xl[2][NVR];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int it = it0 + q * NW;
            if (it >= n_items) break;  // wave-uniform
            const int ex = it / kParts, part = it % kParts;
            const uint4* wq = reinterpret_cast<const uint4*>(ro.router_cm + (size_t)ex * D);
#pragma unroll
            for (int r = 0; r < NVR; ++r) {
                w[q][r] = wq[(part * NVR + r) * kWave + lane];
                xl[q][r] = xp4[(part * NVR + r) * kWave + lane];
            }
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (it0 + q * NW >= n_items) break;
            float acc = 0.0f;
#pragma unroll
            for (int r = 0; r < NVR; ++r) {
                acc = dot2(xl[q][r].x, w[q][r].x, acc);
                acc = dot2(xl[q][r].y, w[q][r].y, acc);
                acc = dot2(xl[q][r].z, w[q][r].z, acc);
                acc = dot2(xl[q][r].w, w[q][r].w, acc);
            }
            acc = group_reduce_sum_to_last<64>(acc);
            if (lane == kWave - 1 && it0 + q * NW < n_items) plog[it0 + q * NW] = acc;
        }
    }
}

}  // namespace floe
