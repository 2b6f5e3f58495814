// S1: router (the paper only says that a router picks the activated experts of each MoE layer, Sec. 3.3;
// the arithmetic is the usual softmax-top-k of the models it evaluates): logits = x . W_r, softmax with the
// maximum subtracted, top_k by probability with ties to the lower expert id, optional renormalisation.
// One workgroup per token writes the task table the later kernels index: task q = token * slots + slot,
// slots 0..top_k-1 routed (descending probability), then the n_shared always-on experts with weight 1.
#include "floe_dev.h"
#include "launch.h"
#include "route.h"

namespace floe {

constexpr int kMaxExperts = 1024;

// All loads of a dot product are in flight together: a lane fetches its 16-byte pieces of x once
// (up to 16 of them, d <= 8192) and of the current expert row, then reduces with packed dot products.
__global__ __launch_bounds__(256) void router_kernel(RouterArgs a) {
    __shared__ float prob[kMaxExperts];
    __shared__ int sel_id[64];
    __shared__ float sel_w[64];
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int d = a.d;
    const int slots = a.top_k + a.n_shared;
    const h16* xt = a.x + (size_t)t * d;
    const int nvec = d / 512;  // 16-byte pieces per lane (d % 512 == 0, d <= 8192)
    if (a.top_k > 0) {
        uint4 xv[16];
        const uint4* xp = reinterpret_cast<const uint4*>(xt);
#pragma unroll
        for (int r = 0; r < 16; ++r) xv[r] = r < nvec ? xp[r * kWave + lane] : make_uint4(0u, 0u, 0u, 0u);
        for (int e = wave; e < a.n_experts; e += 4) {
            const uint4* wp = reinterpret_cast<const uint4*>(a.router_cm + (size_t)e * d);
            uint4 w[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) w[r] = r < nvec ? wp[r * kWave + lane] : make_uint4(0u, 0u, 0u, 0u);
            float acc = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc = dot2(xv[r].x, w[r].x, acc);
                acc = dot2(xv[r].y, w[r].y, acc);
                acc = dot2(xv[r].z, w[r].z, acc);
                acc = dot2(xv[r].w, w[r].w, acc);
            }
            acc = wave_allreduce_sum(acc);
            if (lane == 0) prob[e] = acc;
        }
    }
    __syncthreads();
    if (tid == 0) route_select(prob, a.n_experts, a.top_k, a.n_shared, a.renormalize, sel_id, sel_w);
    __syncthreads();
    // one thread per slot resolves the expert: its pointers, weight and threshold go to the task table
    if (tid < slots) {
        const int e = sel_id[tid];
        const int q = t * slots + tid;
        a.task_expert[q] = e;
        a.task_weight[q] = sel_w[tid];
        a.task_tau[q] = a.tau[(size_t)t * a.tau_stride_t + e];
        a.task_table[q] = a.table[e];
    }
}

hipError_t launch_router(const RouterArgs& a, int T, hipStream_t stream) {
    if (T == 0) return hipSuccess;
    router_kernel<<<dim3(T), dim3(256), 0, stream>>>(a);
    return hipGetLastError();
}

__global__ void stats_kernel(const int32_t* task_expert, const int32_t* count, int count_parts,
                             const float* task_weight, SlotStat* stats, int n_tasks) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_tasks) return;
    SlotStat s;
    s.expert = task_expert[q];
    if (count_parts > 0) {
        int c = 0;
        for (int b = 0; b < count_parts; ++b) c += count[(size_t)q * count_parts + b];
        s.count = c;
    } else {
        s.count = count[q];
    }
    s.weight = task_weight[q];
    s.pad = 0;
    stats[q] = s;
}

hipError_t launch_stats(const int32_t* task_expert, const int32_t* count, int count_parts, const float* task_weight,
                        SlotStat* stats, int n_tasks, hipStream_t stream) {
    if (n_tasks == 0) return hipSuccess;
    stats_kernel<<<dim3((n_tasks + 255) / 256), dim3(256), 0, stream>>>(task_expert, count, count_parts, task_weight,
                                                                        stats, n_tasks);
    return hipGetLastError();
}

}  // namespace floe
