// S4 + S5: gathered gate GEMV with fused SiLU and the product with v, then the gathered down GEMV
// (Alg. 1 lines 4-5), reading only the compact [gate | down] chunks (Sec. 3.4.2) of the selected channels.
//
// Work split: a wave owns whole channels.  For channel j it streams the d fp16 numbers of the gate
// column (128-bit loads, the whole wave covers 1 KiB per load), reduces x . gate across the wave,
// forms h = SiLU(g) * v_j * scale, and adds h * (down row) into d/64 fp32 accumulators per lane.
// Both rows of a channel are requested before either is used.  The waves of a workgroup then add their
// accumulators through LDS and the workgroup stores one partial y; S6 adds the partials.
#include "floe_dev.h"
#include "launch.h"

namespace floe {

template <int NV>  // d = 512 * NV
__global__ __launch_bounds__(256) void gate_down_kernel(TaskMap map, int staged, int gd_rows,
                                                        const h16* __restrict__ x, const float* __restrict__ v,
                                                        const int32_t* __restrict__ idx,
                                                        const int32_t* __restrict__ count,
                                                        const float* __restrict__ task_scale,
                                                        float* __restrict__ partial, int f) {
    constexpr int d = 512 * NV;
    extern __shared__ float red[];  // [4][d]
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int task = blockIdx.y;
    const int t = task / map.slots;
    const DevExpert e = task_expert_of(map, task);
    const float out_scale = task_scale ? task_scale[task] : 1.0f;
    int K = count[task];
    K = min(K, staged ? gd_rows : f);
    const float* vt = v + (size_t)task * f;
    const int32_t* it = idx + (size_t)task * f;

    uint4 xr[NV];
    {
        const uint4* xp = reinterpret_cast<const uint4*>(x + (size_t)t * d);
#pragma unroll
        for (int r = 0; r < NV; ++r) xr[r] = xp[r * kWave + lane];
    }
    float acc[NV * 8];
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) acc[i] = 0.0f;

    const int nw = gridDim.x * 4;
    for (int k = blockIdx.x * 4 + wave; k < K; k += nw) {
        const int j = it[k];
        if ((unsigned)j >= (unsigned)f) continue;  // a caller-supplied list may hold junk: never leave the matrix
        const size_t row = staged ? (size_t)k : (size_t)j;
        const uint4* gp = reinterpret_cast<const uint4*>(e.gd + row * 2 * d);
        const uint4* dp = gp + d / 8;
        uint4 gv[NV], dv[NV];
#pragma unroll
        for (int r = 0; r < NV; ++r) gv[r] = gp[r * kWave + lane];
#pragma unroll
        for (int r = 0; r < NV; ++r) dv[r] = dp[r * kWave + lane];
        const float vj = vt[j];
        float g = 0.0f;
#pragma unroll
        for (int r = 0; r < NV; ++r) {
            g = dot2(xr[r].x, gv[r].x, g);
            g = dot2(xr[r].y, gv[r].y, g);
            g = dot2(xr[r].z, gv[r].z, g);
            g = dot2(xr[r].w, gv[r].w, g);
        }
        g = wave_allreduce_sum(g);
        const float h = silu(g) * vj * out_scale;
#pragma unroll
        for (int r = 0; r < NV; ++r) {
            const uint32_t wds[4] = {dv[r].x, dv[r].y, dv[r].z, dv[r].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const h16x2 p = as_h2(wds[q]);
                acc[r * 8 + 2 * q + 0] = fmaf(h, (float)p.x, acc[r * 8 + 2 * q + 0]);
                acc[r * 8 + 2 * q + 1] = fmaf(h, (float)p.y, acc[r * 8 + 2 * q + 1]);
            }
        }
    }

    // lane holds columns r*512 + lane*8 + e  (e < 8) of its wave's partial y
#pragma unroll
    for (int r = 0; r < NV; ++r) {
        float4* dst = reinterpret_cast<float4*>(red + (size_t)wave * d + r * 512 + lane * 8);
        dst[0] = make_float4(acc[r * 8 + 0], acc[r * 8 + 1], acc[r * 8 + 2], acc[r * 8 + 3]);
        dst[1] = make_float4(acc[r * 8 + 4], acc[r * 8 + 5], acc[r * 8 + 6], acc[r * 8 + 7]);
    }
    __syncthreads();
    float4* out = reinterpret_cast<float4*>(partial + ((size_t)task * gridDim.x + blockIdx.x) * d);
    const float4* r0 = reinterpret_cast<const float4*>(red);
    for (int i = tid; i < d / 4; i += 256) {
        float4 a = r0[i], b = r0[d / 4 + i], c = r0[2 * (d / 4) + i], e4 = r0[3 * (d / 4) + i];
        out[i] = make_float4((a.x + b.x) + (c.x + e4.x), (a.y + b.y) + (c.y + e4.y), (a.z + b.z) + (c.z + e4.z),
                             (a.w + b.w) + (c.w + e4.w));
    }
}

int gd_blocks(int n_tasks, int f) {
    if (n_tasks <= 0) return 1;
    int nblk = kNumCU / n_tasks;
    nblk = nblk < 1 ? 1 : nblk;
    nblk = nblk > kNumCU ? kNumCU : nblk;
    const int by_f = (f + 3) / 4;  // never more waves than channels
    nblk = nblk > by_f ? by_f : nblk;
    return nblk < 1 ? 1 : nblk;
}

template <int NV>
static hipError_t launch_nv(const TaskMap& map, int staged, int gd_rows, const h16* x, const float* v,
                            const int32_t* idx, const int32_t* count, const float* task_scale, float* partial, int f,
                            int n_tasks, int nblk, hipStream_t stream) {
    constexpr size_t lds = (size_t)4 * 512 * NV * sizeof(float);
    static bool attr_set = false;
    if (!attr_set && lds > 48 * 1024) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&gate_down_kernel<NV>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (rc != hipSuccess) return rc;
        attr_set = true;
    }
    gate_down_kernel<NV><<<dim3(nblk, n_tasks), dim3(256), lds, stream>>>(map, staged, gd_rows, x, v, idx, count,
                                                                         task_scale, partial, f);
    return hipGetLastError();
}

hipError_t launch_gate_down(const TaskMap& map, int staged, int gd_rows, const h16* x, const float* v,
                            const int32_t* idx, const int32_t* count, const float* task_scale, float* partial, int d,
                            int f, int n_tasks, int nblk, hipStream_t stream) {
    if (n_tasks == 0) return hipSuccess;
#define FLOE_NV_CASE(N) \
    case N: return launch_nv<N>(map, staged, gd_rows, x, v, idx, count, task_scale, partial, f, n_tasks, nblk, stream);
    switch (d / 512) {
        FLOE_NV_CASE(1) FLOE_NV_CASE(2) FLOE_NV_CASE(3) FLOE_NV_CASE(4) FLOE_NV_CASE(5) FLOE_NV_CASE(6)
        FLOE_NV_CASE(7) FLOE_NV_CASE(8) FLOE_NV_CASE(9) FLOE_NV_CASE(10) FLOE_NV_CASE(11) FLOE_NV_CASE(12)
        FLOE_NV_CASE(13) FLOE_NV_CASE(14) FLOE_NV_CASE(15) FLOE_NV_CASE(16)
        default: return hipErrorInvalidValue;
    }
#undef FLOE_NV_CASE
}

// ---------------------------------------------------------------------------------------------------
// S6: sum the partial results of every (slot, block) of a token, fold into y_acc and / or round to fp16.
// A workgroup owns 64 output columns of one token: 16 threads (one float4 each) cover the columns,
// the 16 thread rows split the partials between them and meet in LDS.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ partial, int d, int per_token,
                                                      float* __restrict__ y_acc, h16* __restrict__ y_half) {
    __shared__ float4 red[16][16];
    const int t = blockIdx.y;
    const int cg = threadIdx.x & 15, pg = threadIdx.x >> 4;
    const int c4 = blockIdx.x * 16 + cg;  // column / 4   (d % 64 == 0)
    const float4* p = reinterpret_cast<const float4*>(partial + (size_t)t * per_token * d) + c4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int b = pg; b < per_token; b += 16) {
        const float4 a = p[(size_t)b * (d / 4)];
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
    red[pg][cg] = s;
    __syncthreads();
    if (pg != 0) return;
#pragma unroll
    for (int r = 1; r < 16; ++r) {
        const float4 a = red[r][cg];
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
    if (y_acc) {
        float4* y = reinterpret_cast<float4*>(y_acc + (size_t)t * d) + c4;
        float4 o = *y;
        o.x += s.x; o.y += s.y; o.z += s.z; o.w += s.w;
        *y = o;
    }
    if (y_half) {
        h16* y = y_half + (size_t)t * d + c4 * 4;
        h16x2 lo = {(h16)s.x, (h16)s.y}, hi = {(h16)s.z, (h16)s.w};
        *reinterpret_cast<uint2*>(y) = make_uint2(as_u32(lo), as_u32(hi));
    }
}

hipError_t launch_combine(const float* partial, int d, int T, int slots, int nblk, float* y_acc, h16* y_half,
                          hipStream_t stream) {
    if (T == 0) return hipSuccess;
    dim3 grid(d / 64, T);
    combine_kernel<<<grid, dim3(256), 0, stream>>>(partial, d, slots * nblk, y_acc, y_half);
    return hipGetLastError();
}

}  // namespace floe
