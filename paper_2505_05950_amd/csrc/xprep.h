// Activation preparation for the packed-fp16 dequant GEMV (see up_gemv.hip).
//
// A lane owns one "unit" of 64 consecutive codes of a channel and the 64 activations that go with
// them.  Codes are never turned into numbers one by one.  A bit field of a code word that sits at
// mantissa bits [p, p+b) of a 16-bit half is OR-ed into 0x3C00, which reads as the fp16 number
// 1 + q * 2^(p-10); the activation that meets it is pre-multiplied by c = 2^(10-p), so one packed
// dot product adds c*x + x*q to an fp32 accumulator.  sum(c*x) is taken off once per unit.
// This header turns the lane's 64 activations into the 32 fp16 pairs (already times c) that the
// extraction order of each bit width wants, and into the two sums per half unit (32 codes).
#pragma once

#include "floe_dev.h"

namespace floe {

__device__ __forceinline__ float unit_amax(const uint32_t (&raw)[32]) {
    float amax = 0.0f;
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        const h16x2 p = as_h2(raw[r]);
        amax = fmaxf(amax, fmaxf(fabsf((float)p.x), fabsf((float)p.y)));
    }
    return amax;
}

// largest multiplier c the extraction of each bit width uses
template <int BITS> struct PackedTraits;
template <> struct PackedTraits<2> { static constexpr int kWords = 4; static constexpr int kLog2MaxC = 6; };
template <> struct PackedTraits<3> { static constexpr int kWords = 6; static constexpr int kLog2MaxC = 7; };
template <> struct PackedTraits<4> { static constexpr int kWords = 8; static constexpr int kLog2MaxC = 8; };

// power-of-two down-scaling exponent: x' = x * 2^-down keeps maxc * |x'| below 2^15 in fp16
template <int BITS>
__device__ __forceinline__ int xprep_down(float token_amax) {
    constexpr int kKeepBelow = 15 - PackedTraits<BITS>::kLog2MaxC;  // |x'| < 2^kKeepBelow
    const float lim = (float)(1 << (kKeepBelow - 1));
    return (token_amax >= lim && token_amax < 3.0e38f) ? ilogbf(token_amax) - (kKeepBelow - 1) : 0;
}

// activation i of the unit (0..63) from the raw registers: raw[r] = (x[2r], x[2r+1])
__device__ __forceinline__ uint32_t pair_of(const uint32_t (&raw)[32], int lo, int hi) {
    const uint32_t A = raw[lo >> 1], B = raw[hi >> 1];
    const uint32_t a16 = (lo & 1) ? (A >> 16) : (A & 0xFFFFu);
    const uint32_t b16 = (hi & 1) ? (B >> 16) : (B & 0xFFFFu);
    return a16 | (b16 << 16);
}

// Order of the 32 registers and their multipliers (h = half unit 0/1, i.e. codes 32h .. 32h+31):
//  INT2: word w (16 codes) gives registers 8w+m, m<8: codes (16w+m, 16w+m+8), c = {64,16,64,16,4,64,16,4}
//  INT4: word w (8 codes)  gives registers 4w+m, m<4: codes (8w+m, 8w+m+4),   c = {64,64,256,16}
//  INT3: half h (96 bits) gives registers 16h + 5k + i for the three 10-code chunks k<3, i<5:
//        codes (32h+10k+i, 32h+10k+i+5), c = {128,128,16,128,16}; register 16h+15: codes (32h+30, 32h+31), c = 16
template <int BITS>
__device__ __forceinline__ void unit_layout(int reg, int& lo, int& hi, float& c) {
    if (BITS == 2) {
        const int w = reg >> 3, m = reg & 7;
        const float cm[8] = {64.f, 16.f, 64.f, 16.f, 4.f, 64.f, 16.f, 4.f};
        lo = 16 * w + m; hi = lo + 8; c = cm[m];
    } else if (BITS == 4) {
        const int w = reg >> 2, m = reg & 3;
        const float cm[4] = {64.f, 64.f, 256.f, 16.f};
        lo = 8 * w + m; hi = lo + 4; c = cm[m];
    } else {
        const int h = reg >> 4, r = reg & 15;
        if (r == 15) { lo = 32 * h + 30; hi = lo + 1; c = 16.f; }
        else {
            const int k = r / 5, i = r % 5;
            const float cm[5] = {128.f, 128.f, 16.f, 128.f, 16.f};
            lo = 32 * h + 10 * k + i; hi = lo + 5; c = cm[i];
        }
    }
}

// xs[32]: prepared pairs;  Xoff[h] = sum of c*x', Xg[h] = sum of x' over half unit h
template <int BITS>
__device__ __forceinline__ void unit_prepare(const uint32_t (&raw)[32], int down, uint32_t (&xs)[32], float (&Xoff)[2],
                                             float (&Xg)[2]) {
    const h16 pscale = (h16)ldexpf(1.0f, -down);
    const h16x2 ones = {(h16)1.0f, (h16)1.0f};
    Xg[0] = Xg[1] = Xoff[0] = Xoff[1] = 0.0f;
#pragma unroll
    for (int reg = 0; reg < 32; ++reg) {
        int lo, hi;
        float c;
        unit_layout<BITS>(reg, lo, hi, c);
        const int h = reg >> 4;  // every layout keeps registers 0..15 in the first half unit
        h16x2 p = as_h2(pair_of(raw, lo, hi)) * (h16x2){pscale, pscale};
        Xg[h] = __builtin_amdgcn_fdot2(p, ones, Xg[h], false);
        p = p * (h16x2){(h16)c, (h16)c};
        Xoff[h] = __builtin_amdgcn_fdot2(p, ones, Xoff[h], false);
        xs[reg] = as_u32(p);
    }
}

// sum over half unit h of x' * q (plus the c*x' part, which the caller removes with Xoff[h])
// cw: the unit's code words (PackedTraits<BITS>::kWords of them), magic = 0x3C003C00 held in a VGPR.
template <int BITS>
__device__ __forceinline__ float half_unit_dot(const uint32_t* cw, const uint32_t (&xs)[32], int h, uint32_t magic) {
    float dot = 0.0f;
    if (BITS == 2) {
#pragma unroll
        for (int w = 2 * h; w < 2 * h + 2; ++w) {
            const uint32_t W = cw[w], a = W << 4, b = W >> 6;
            dot = dot2(xs[8 * w + 0], and_or(a, 0x00300030u, magic), dot);
            dot = dot2(xs[8 * w + 1], and_or(a, 0x00C000C0u, magic), dot);
            dot = dot2(xs[8 * w + 2], and_or(W, 0x00300030u, magic), dot);
            dot = dot2(xs[8 * w + 3], and_or(W, 0x00C000C0u, magic), dot);
            dot = dot2(xs[8 * w + 4], and_or(W, 0x03000300u, magic), dot);
            dot = dot2(xs[8 * w + 5], and_or(b, 0x00300030u, magic), dot);
            dot = dot2(xs[8 * w + 6], and_or(b, 0x00C000C0u, magic), dot);
            dot = dot2(xs[8 * w + 7], and_or(b, 0x03000300u, magic), dot);
        }
    } else if (BITS == 4) {
#pragma unroll
        for (int w = 4 * h; w < 4 * h + 4; ++w) {
            const uint32_t W = cw[w], a = W << 4, b = W >> 6;
            dot = dot2(xs[4 * w + 0], and_or(a, 0x00F000F0u, magic), dot);  // code 0 -> bits [4,8)
            dot = dot2(xs[4 * w + 1], and_or(W, 0x00F000F0u, magic), dot);  // code 1 at bits [4,8)
            dot = dot2(xs[4 * w + 2], and_or(b, 0x003C003Cu, magic), dot);  // code 2 -> bits [2,6)
            dot = dot2(xs[4 * w + 3], and_or(b, 0x03C003C0u, magic), dot);  // code 3 -> bits [6,10)
        }
    } else {
        const uint32_t w0 = cw[3 * h], w1 = cw[3 * h + 1], w2 = cw[3 * h + 2];
        const uint32_t chunk[3] = {w0, __builtin_amdgcn_alignbit(w1, w0, 30), __builtin_amdgcn_alignbit(w2, w1, 28)};
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            // codes 0..4 of the chunk in the low half, codes 5..9 in the high half, 3 bits apart
            const uint32_t t = (chunk[k] & 0x7FFFu) | ((chunk[k] << 1) & 0x7FFF0000u);
            const uint32_t a = t << 3, b = t >> 6;
            const int r = 16 * h + 5 * k;
            dot = dot2(xs[r + 0], and_or(a, 0x00380038u, magic), dot);  // code 0 -> bits [3,6)
            dot = dot2(xs[r + 1], and_or(t, 0x00380038u, magic), dot);  // code 1 at bits [3,6)
            dot = dot2(xs[r + 2], and_or(t, 0x01C001C0u, magic), dot);  // code 2 at bits [6,9)
            dot = dot2(xs[r + 3], and_or(b, 0x00380038u, magic), dot);  // code 3 -> bits [3,6)
            dot = dot2(xs[r + 4], and_or(b, 0x01C001C0u, magic), dot);  // code 4 -> bits [6,9)
        }
        // codes 30, 31: bits 26..28 and 29..31 of the last word -> bits [6,9) of the low and high half
        const uint32_t tail = ((w2 >> 20) & 0x000001C0u) | ((w2 >> 7) & 0x01C00000u);
        dot = dot2(xs[16 * h + 15], tail | magic, dot);
    }
    return dot;
}

}  // namespace floe
