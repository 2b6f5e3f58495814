// Pieces shared by the kernels that stream packed codes (up_gemv.hip, fused_layer.hip): a lane's load of one
// 64-code unit with its scale / zero, and the value of a channel from it.
#pragma once

#include "floe_dev.h"
#include "xprep.h"

namespace floe {

template <int BITS>
__device__ __forceinline__ void load_unit(const uint32_t* __restrict__ codes, size_t unit_index, uint32_t* cw) {
    constexpr int W = PackedTraits<BITS>::kWords;
    const uint32_t* p = codes + unit_index * W;
    if (BITS == 2) {
        const uint4 q = gload16(p);
        cw[0] = q.x; cw[1] = q.y; cw[2] = q.z; cw[3] = q.w;
    } else if (BITS == 4) {
        const uint4 q0 = gload16(p), q1 = gload16(p + 4);
        cw[0] = q0.x; cw[1] = q0.y; cw[2] = q0.z; cw[3] = q0.w;
        cw[4] = q1.x; cw[5] = q1.y; cw[6] = q1.z; cw[7] = q1.w;
    } else {  // 24 bytes, 8-byte aligned
        const uint2 q0 = gload8(p), q1 = gload8(p + 2), q2 = gload8(p + 4);
        cw[0] = q0.x; cw[1] = q0.y; cw[2] = q1.x; cw[3] = q1.y; cw[4] = q2.x; cw[5] = q2.y;
    }
}

template <int BITS, int UPC, bool G32>
struct UnitLoad {  // one pass of a lane: the unit's code words and its scale / zero
    uint32_t cw[PackedTraits<BITS>::kWords];
    uint32_t s, z;  // groups of 32: the unit's two scales / zeros
    h16 sh, zh;     // larger groups: its one scale / zero, kept as a half (a 16-bit load leaves the rest of the
                    // register alone, so widening it to 32 bits would be an instruction that waits for the load)
    __device__ __forceinline__ void issue(const DevExpert& e, int j, int u, int G, int gshift) {
        load_unit<BITS>(e.codes, (size_t)j * UPC + u, cw);
        issue_meta(e, j, u, G, gshift);
    }
    // the same with the lane's part of the address precomputed: lane_scale / lane_zero point at the lane's entry of
    // channel 0 and row is the channel's offset in entries (a scalar where the channel is the same for every lane)
    __device__ __forceinline__ void issue_meta_at(const h16* lane_scale, const h16* lane_zero, size_t row) {
        if (G32) {
            s = gload4(lane_scale + row);
            z = gload4(lane_zero + row);
        } else {
            sh = gloadh(lane_scale + row);
            zh = gloadh(lane_zero + row);
        }
    }
    __device__ __forceinline__ void issue_meta(const DevExpert& e, int j, int u, int G, int gshift) {
        if (G32) {
            const size_t mi = (size_t)j * G + 2 * u;  // even index: 4-byte aligned
            s = gload4(e.scale + mi);
            z = gload4(e.zero + mi);
        } else {
            const size_t mi = (size_t)j * G + ((u * 64) >> gshift);
            sh = gloadh(e.scale + mi);
            zh = gloadh(e.zero + mi);
        }
    }
};


// s * (sum x'q - Xoff - z * Xg) of a lane's unit: the lane's share of v_j (before the sum over the channel's lanes)
template <int BITS, int UPC, bool G32>
__device__ __forceinline__ float unit_value(const UnitLoad<BITS, UPC, G32>& L, const uint32_t (&xs)[32],
                                            const float (&Xoff)[2], const float (&Xg)[2], uint32_t magic) {
    const float dot0 = half_unit_dot<BITS>(L.cw, xs, 0, magic);
    const float dot1 = half_unit_dot<BITS>(L.cw, xs, 1, magic);
    if (G32) {
        const h16x2 s2 = as_h2(L.s), z2 = as_h2(L.z);
        return (float)s2.x * fmaf(-(float)z2.x, Xg[0], dot0 - Xoff[0]) + (float)s2.y * fmaf(-(float)z2.y, Xg[1], dot1 - Xoff[1]);
    }
    const float sc = (float)L.sh, z = (float)L.zh;
    return sc * fmaf(-z, Xg[0] + Xg[1], (dot0 + dot1) - (Xoff[0] + Xoff[1]));
}

}  // namespace floe
