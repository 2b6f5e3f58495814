// Activation preparation for the packed-fp16 INT2 GEMV (see up_gemv.hip): a lane that owns the 64
// activations of one "unit" turns them into 32 fp16 pairs, pre-multiplied by the constants that undo
// the position of each 2-bit field inside the fp16 mantissa.
#pragma once

#include "floe_dev.h"

namespace floe {

// Prepared activations of T tokens in HBM (written by the router kernel for the layer path).
struct XPrep {
    uint4* xs;     // [T][8][UPC] : register r4 (0..7) of unit u at xs[(t*8 + r4)*UPC + u]
    float* xoff;   // [T][UPC]    : sum of c*x over the unit
    float* xg;     // [T][UPC]    : sum of x over the unit
    float* inv_p;  // [T]         : 2^down, multiplies v at the end
};

__device__ __forceinline__ float unit_amax(const uint32_t (&raw)[32]) {
    float amax = 0.0f;
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        const h16x2 p = as_h2(raw[r]);
        amax = fmaxf(amax, fmaxf(fabsf((float)p.x), fabsf((float)p.y)));
    }
    return amax;
}

// power-of-two down-scaling exponent that keeps 64 * |x| below 2^15 in fp16
__device__ __forceinline__ int xprep_down(float token_amax) {
    return (token_amax >= 256.0f && token_amax < 3.0e38f) ? ilogbf(token_amax) - 7 : 0;
}

// raw[r] = (x[2r], x[2r+1]) of the unit.  Output register 8*w + m pairs activation 16w+m (low half)
// with activation 16w+m+8 (high half), both times c_m, c = {64,16,64,16,4,64,16,4}.
__device__ __forceinline__ void unit_prepare(const uint32_t (&raw)[32], int down, uint32_t (&xs)[32], float& Xoff,
                                             float& Xg) {
    const h16 pscale = (h16)ldexpf(1.0f, -down);
    const h16x2 ones = {(h16)1.0f, (h16)1.0f};
    const float cm[8] = {64.f, 16.f, 64.f, 16.f, 4.f, 64.f, 16.f, 4.f};
    Xg = 0.0f;
    Xoff = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            const uint32_t A = raw[8 * w + m / 2], B = raw[8 * w + 4 + m / 2];
            const uint32_t pr = (m & 1) ? ((A >> 16) | (B & 0xFFFF0000u)) : ((A & 0xFFFFu) | (B << 16));
            h16x2 p = as_h2(pr) * (h16x2){pscale, pscale};
            Xg = __builtin_amdgcn_fdot2(p, ones, Xg, false);
            p = p * (h16x2){(h16)cm[m], (h16)cm[m]};
            Xoff = __builtin_amdgcn_fdot2(p, ones, Xoff, false);
            xs[8 * w + m] = as_u32(p);
        }
    }
}

}  // namespace floe
