// S0: asymmetric uniform group quantizer for the up projection (paper Sec. 3.2.2).
// Bit-exact contract (stated in include/floe.h): strict IEEE binary32, one rounding per operation,
// no fused multiply-add, correctly rounded division, round-half-even to integer and to fp16.
#include "floe_dev.h"
#include "launch.h"

namespace floe {

#pragma clang fp contract(off)

// One workgroup per channel.  A thread owns 8 consecutive weights (one 16-byte load); the g/8 lanes
// of a group find min/max with xor-shuffles, every lane derives the same (scale, zero), computes its
// 8 codes and parks them in LDS as bytes; then each thread assembles whole 32-bit words of the
// channel's little-endian bit stream and stores them coalesced.
template <int BITS>
__global__ __launch_bounds__(256) void quantize_kernel(const h16* __restrict__ w, uint32_t* __restrict__ codes,
                                                       h16* __restrict__ scale, h16* __restrict__ zero, int d,
                                                       int group) {
    constexpr int kChunk = 256 * 8;  // weights handled per loop trip
    __shared__ uint8_t q_lds[kChunk];
    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    const int lanes_per_group = group / 8;  // power of two in [4, 32]
    const int G = d / group;
    const int wpc = d * BITS / 32;
    const float qmax = (float)((1 << BITS) - 1);
    const h16* wj = w + (size_t)j * d;

    for (int base = 0; base < d; base += kChunk) {
        const int i0 = base + tid * 8;
        const bool live = i0 < d;  // d % 8 == 0, so a thread is entirely in or out
        float a[8];
        if (live) {
            uint4 raw = *reinterpret_cast<const uint4*>(wj + i0);
            const h16* hp = reinterpret_cast<const h16*>(&raw);
#pragma unroll
            for (int e = 0; e < 8; ++e) a[e] = (float)hp[e];
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) a[e] = 0.0f;
        }
        float mn = a[0], mx = a[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) {
            mn = fminf(mn, a[e]);
            mx = fmaxf(mx, a[e]);
        }
        // groups are aligned to lanes_per_group lanes; dead lanes only ever pair with dead lanes
        // because d is a multiple of the group length
        for (int o = 1; o < lanes_per_group; o <<= 1) {
            mn = fminf(mn, __shfl_xor(mn, o, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, o, kWave));
        }
        const float range = mx - mn;
        const float s32 = range / qmax;
        h16 sh = (h16)s32;  // v_cvt_f16_f32, round to nearest even
        const float S = (float)sh;
        const bool degenerate = !(mx > mn) || !(S >= 6.103515625e-05f) || __builtin_isinf(S);
        h16 zh;
        uint32_t q[8];
        if (degenerate) {
            sh = (h16)1.0f;
            zh = (h16)(-mn);
#pragma unroll
            for (int e = 0; e < 8; ++e) q[e] = 0;
        } else {
            float z32 = (-mn) / S;
            z32 = fminf(fmaxf(z32, -65504.0f), 65504.0f);
            zh = (h16)z32;
            const float Z = (float)zh;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float t = a[e] / S;
                float u = t + Z;
                float r = __builtin_rintf(u);
                r = fminf(fmaxf(r, 0.0f), qmax);
                q[e] = (uint32_t)r;
            }
        }
        if (live) {
            uint32_t lo = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
            uint32_t hi = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
            *reinterpret_cast<uint2*>(&q_lds[tid * 8]) = make_uint2(lo, hi);
            if ((i0 % group) == 0) {
                scale[(size_t)j * G + i0 / group] = sh;
                zero[(size_t)j * G + i0 / group] = zh;
            }
        }
        __syncthreads();
        // pack: word ww of this chunk holds bits [32 ww, 32 ww + 32) of the chunk's bit stream
        const int chunk_len = min(kChunk, d - base);
        const int chunk_words = chunk_len * BITS / 32;  // chunk_len % 32 == 0
        for (int ww = tid; ww < chunk_words; ww += 256) {
            const int bit0 = ww * 32;
            const int first = bit0 / BITS;
            const int last = (bit0 + 31) / BITS;
            uint32_t word = 0;
            for (int c = first; c <= last; ++c) {
                const int sh_bits = c * BITS - bit0;
                const uint32_t qq = q_lds[c];
                word |= sh_bits >= 0 ? (qq << sh_bits) : (qq >> (-sh_bits));
            }
            codes[(size_t)j * wpc + base * BITS / 32 + ww] = word;
        }
        __syncthreads();
    }
}

hipError_t launch_quantize(const h16* w, uint32_t* codes, h16* scale, h16* zero, int d, int f, int bits, int group,
                           hipStream_t stream) {
    if (f == 0) return hipSuccess;
    dim3 grid(f), block(256);
    switch (bits) {
        case 1: quantize_kernel<1><<<grid, block, 0, stream>>>(w, codes, scale, zero, d, group); break;
        case 8: quantize_kernel<8><<<grid, block, 0, stream>>>(w, codes, scale, zero, d, group); break;
        case 2: quantize_kernel<2><<<grid, block, 0, stream>>>(w, codes, scale, zero, d, group); break;
        case 3: quantize_kernel<3><<<grid, block, 0, stream>>>(w, codes, scale, zero, d, group); break;
        default: quantize_kernel<4><<<grid, block, 0, stream>>>(w, codes, scale, zero, d, group); break;
    }
    return hipGetLastError();
}

}  // namespace floe
