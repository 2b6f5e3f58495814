// The other two candidates for sparsification of Sec. 3.2.1: the sparsity function S_t (Eq. 5) applied to
// a_gate = SiLU(x . W_gate) or to a_down = a_gate * a_up (Eq. 3-4) instead of a_up, inside the expert forward of Eq. 1.
// They exist to show, on this machine, what the paper argues in Sec. 3.2.1: only thresholding a_up saves the traffic
// of BOTH remaining matrices.  With a_gate or a_down the whole gate projection has to be read before a single channel
// can be dropped (f * 2d bytes), and only the down rows of the dropped channels are saved.
//
//   gate_dense_kernel   a wave per channel: the whole gate column (1 KiB per wave instruction), packed dot products,
//                       DPP reduction; writes act[j] (the activation that is compared with t) and h[j] = a_gate_j * a_up_j
//   down_rows_kernel    y partial = sum over the kept channels of h[j] * W_down[j, :] (the down half of each chunk only)
// Selection in between is the stand-alone S3 kernel (select.hip); the partial results are added by combine_kernel.
#include "floe_dev.h"
#include "launch.h"

namespace floe {

template <int NV>  // d = 512 * NV
__global__ __launch_bounds__(256) void gate_dense_kernel(const h16* __restrict__ gd, const h16* __restrict__ x,
                                                         const float* __restrict__ v, int which, int f,
                                                         float* __restrict__ act, float* __restrict__ hval) {
    constexpr int d = 512 * NV;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.y;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
    uint4 xr[NV];
    {
        const uint4* xp = reinterpret_cast<const uint4*>(x + (size_t)t * d);
#pragma unroll
        for (int c = 0; c < NV; ++c) xr[c] = xp[c * kWave + lane];
    }
    const float* vt = v + (size_t)t * f;
    // two columns in flight per wave
    for (int j0 = gw; j0 < f; j0 += 2 * nw) {
        const int j1 = j0 + nw < f ? j0 + nw : j0;
        const uint4* g0 = reinterpret_cast<const uint4*>(gd + (size_t)j0 * 2 * d);
        const uint4* g1 = reinterpret_cast<const uint4*>(gd + (size_t)j1 * 2 * d);
        uint4 q0[NV], q1[NV];
#pragma unroll
        for (int c = 0; c < NV; ++c) q0[c] = g0[c * kWave + lane];
#pragma unroll
        for (int c = 0; c < NV; ++c) q1[c] = g1[c * kWave + lane];
        const float v0 = vt[j0], v1 = vt[j1];
        float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            a0 = dot2(xr[c].x, q0[c].x, a0); a0 = dot2(xr[c].y, q0[c].y, a0);
            a0 = dot2(xr[c].z, q0[c].z, a0); a0 = dot2(xr[c].w, q0[c].w, a0);
            a1 = dot2(xr[c].x, q1[c].x, a1); a1 = dot2(xr[c].y, q1[c].y, a1);
            a1 = dot2(xr[c].z, q1[c].z, a1); a1 = dot2(xr[c].w, q1[c].w, a1);
        }
        a0 = silu(wave_allreduce_sum(a0));
        a1 = silu(wave_allreduce_sum(a1));
        if (lane == 0) {
            const float h0 = a0 * v0, h1 = a1 * v1;
            act[(size_t)t * f + j0] = which == 1 ? a0 : h0;
            hval[(size_t)t * f + j0] = h0;
            if (j1 != j0) {
                act[(size_t)t * f + j1] = which == 1 ? a1 : h1;
                hval[(size_t)t * f + j1] = h1;
            }
        }
    }
}

template <int NV>  // d = 512 * NV; 256 threads, thread owns 16-byte pieces tid, tid + 256, ... of a row
__global__ __launch_bounds__(256) void down_rows_kernel(const h16* __restrict__ gd, const float* __restrict__ hval,
                                                        const int32_t* __restrict__ idx, const int32_t* __restrict__ count,
                                                        const float* __restrict__ out_scale, int f,
                                                        float* __restrict__ partial) {
    constexpr int d = 512 * NV;
    constexpr int VPR = d / 8;               // 16-byte pieces per row
    constexpr int RG = (VPR + 255) / 256;    // pieces per thread per row
    constexpr int B = 8;                     // rows in flight
    __shared__ int jl[B];
    __shared__ float hl[B];
    const int tid = threadIdx.x;
    const int t = blockIdx.y;
    const int K = min(count[t], f);
    const int per = (K + (int)gridDim.x - 1) / (int)gridDim.x;
    const int k0 = min(K, (int)blockIdx.x * per), k1 = min(K, k0 + per);
    const float sc = out_scale ? out_scale[t] : 1.0f;
    float acc[RG * 8];
#pragma unroll
    for (int i = 0; i < RG * 8; ++i) acc[i] = 0.0f;
    for (int kb = k0; kb < k1; kb += B) {
        __syncthreads();  // the previous batch's list is no longer read
        if (tid < B) {
            const int k = kb + tid;
            int j = k < k1 ? idx[(size_t)t * f + k] : -1;
            if ((unsigned)j >= (unsigned)f) j = -1;  // a caller-supplied list may hold junk: never leave the matrix
            jl[tid] = j;
            hl[tid] = j >= 0 ? hval[(size_t)t * f + j] * sc : 0.0f;
        }
        __syncthreads();
        uint4 dv[B][RG];
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const int j = jl[b];
            const uint4* dp = reinterpret_cast<const uint4*>(gd + (size_t)(j < 0 ? 0 : j) * 2 * d + d);
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const int piece = tid + 256 * r;
                dv[b][r] = (j >= 0 && piece < VPR) ? dp[piece] : make_uint4(0u, 0u, 0u, 0u);
            }
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const float h = hl[b];
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const uint32_t wds[4] = {dv[b][r].x, dv[b][r].y, dv[b][r].z, dv[b][r].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const h16x2 p = as_h2(wds[q]);
                    acc[r * 8 + 2 * q + 0] = fmaf(h, (float)p.x, acc[r * 8 + 2 * q + 0]);
                    acc[r * 8 + 2 * q + 1] = fmaf(h, (float)p.y, acc[r * 8 + 2 * q + 1]);
                }
            }
        }
    }
    float* out = partial + ((size_t)t * gridDim.x + blockIdx.x) * d;
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const int piece = tid + 256 * r;
        if (piece < VPR) {
            float4* o4 = reinterpret_cast<float4*>(out + (size_t)piece * 8);
            o4[0] = make_float4(acc[r * 8 + 0], acc[r * 8 + 1], acc[r * 8 + 2], acc[r * 8 + 3]);
            o4[1] = make_float4(acc[r * 8 + 4], acc[r * 8 + 5], acc[r * 8 + 6], acc[r * 8 + 7]);
        }
    }
}

template <int NV>
static hipError_t launch_variant_nv(const h16* gd, const h16* x, const float* v, int which, int f, int T, float* act,
                                    float* hval, hipStream_t stream) {
    const int by_f = (f + 7) / 8;  // at least two columns per wave
    int nb = 2 * num_cus() / (T > 0 ? T : 1);
    nb = nb < 1 ? 1 : (nb > by_f ? by_f : nb);
    gate_dense_kernel<NV><<<dim3(nb, T), dim3(256), 0, stream>>>(gd, x, v, which, f, act, hval);
    return hipGetLastError();
}

hipError_t launch_gate_dense(const h16* gd, const h16* x, const float* v, int which, int d, int f, int T, float* act,
                             float* hval, hipStream_t stream) {
    if (T == 0 || f == 0) return hipSuccess;
    switch (d / 512) {
#define FLOE_NV_CASE(N) case N: return launch_variant_nv<N>(gd, x, v, which, f, T, act, hval, stream);
        FLOE_NV_CASE(1) FLOE_NV_CASE(2) FLOE_NV_CASE(3) FLOE_NV_CASE(4) FLOE_NV_CASE(5) FLOE_NV_CASE(6)
        FLOE_NV_CASE(7) FLOE_NV_CASE(8) FLOE_NV_CASE(9) FLOE_NV_CASE(10) FLOE_NV_CASE(11) FLOE_NV_CASE(12)
        FLOE_NV_CASE(13) FLOE_NV_CASE(14) FLOE_NV_CASE(15) FLOE_NV_CASE(16)
#undef FLOE_NV_CASE
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_down_rows(const h16* gd, const float* hval, const int32_t* idx, const int32_t* count,
                            const float* out_scale, int d, int f, int T, int nblk, float* partial, hipStream_t stream) {
    if (T == 0) return hipSuccess;
    const dim3 grid(nblk, T), block(256);
    switch (d / 512) {
#define FLOE_NV_CASE(N) \
    case N: down_rows_kernel<N><<<grid, block, 0, stream>>>(gd, hval, idx, count, out_scale, f, partial); break;
        FLOE_NV_CASE(1) FLOE_NV_CASE(2) FLOE_NV_CASE(3) FLOE_NV_CASE(4) FLOE_NV_CASE(5) FLOE_NV_CASE(6)
        FLOE_NV_CASE(7) FLOE_NV_CASE(8) FLOE_NV_CASE(9) FLOE_NV_CASE(10) FLOE_NV_CASE(11) FLOE_NV_CASE(12)
        FLOE_NV_CASE(13) FLOE_NV_CASE(14) FLOE_NV_CASE(15) FLOE_NV_CASE(16)
#undef FLOE_NV_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace floe
