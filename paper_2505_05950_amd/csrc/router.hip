// S1: router (the paper only says that a router picks the activated experts of each MoE layer, Sec. 3.3;
// the arithmetic is the usual softmax-top-k of the models it evaluates): logits = x . W_r, softmax with the
// maximum subtracted, top_k by probability with ties to the lower expert id, optional renormalisation.
// One workgroup per token (or, for many experts, two launches: see router_logits_kernel) writes the task table the
// later kernels index: task q = token * slots + slot,
// slots 0..top_k-1 routed (descending probability), then the n_shared always-on experts with weight 1.
#include "floe_dev.h"
#include "launch.h"
#include "route.h"

namespace floe {

constexpr int kMaxExperts = 1024;

// Softmax + top-k for n <= 64 experts on one wave (lane e holds expert e).  Same expf and the same tie rule (lower id)
// as route_select; the sum of the exponentials is a DPP tree instead of that routine's ascending chain (64 dependent
// scalar reads cost more than the rest of the routing together), so weights may differ from it in the last bit.
__device__ __forceinline__ float lane_f(float v, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ void route_select_wave64(float logit, int lane, int n, int top_k, int renormalize, int* sel_id,
                                                    float* sel_w) {
    const bool live = lane < n;
    // maximum: inside the rows of 16 on the DPP path, then over the four rows through scalar registers
    float mx = row16_allreduce_max(live ? logit : -INFINITY);
    mx = fmaxf(fmaxf(lane_f(mx, 0), lane_f(mx, 16)), fmaxf(lane_f(mx, 32), lane_f(mx, 48)));
    const float p = live ? expf(logit - mx) : 0.0f;
    const float sum = wave_allreduce_sum(p);
    float cur = live ? p : -3.0f;
    float sel = 0.0f, my_w = 0.0f;
    int my_id = 0;
    for (int r = 0; r < top_k; ++r) {
        // arg-max with ties to the lower id: (value, id) pairs rotate around each row of 16, then the four row
        // winners (in ascending id order, so a strict comparison keeps the lower id) meet in scalar registers
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
        float wv = lane_f(bv, 0);
        int wi = __builtin_amdgcn_readlane(bi, 0);
#pragma unroll
        for (int row = 1; row < 4; ++row) {
            const float ov = lane_f(bv, 16 * row);
            const int oi = __builtin_amdgcn_readlane(bi, 16 * row);
            if (ov > wv) { wv = ov; wi = oi; }
        }
        const float pw = wv / sum;
        if (lane == r) { my_w = pw; my_id = wi; }
        sel += pw;
        if (lane == wi) cur = -2.0f;  // taken
    }
    if (lane < top_k) {
        sel_id[lane] = my_id;
        sel_w[lane] = renormalize ? my_w / sel : my_w;
    }
}

// logit of expert e for the token whose x pieces the lanes hold, for up to Q experts at a time: all 16-byte pieces of
// the Q rows are requested before the packed dot products run.  Every lane returns the full sums.
template <int NV, int Q>
__device__ __forceinline__ void router_logits(const h16* __restrict__ router_cm, const uint4 (&xv)[NV], int lane,
                                              const int (&e)[Q], float (&out)[Q]) {
    constexpr int d = NV * 512;
    uint4 w[Q][NV];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const uint4* wp = reinterpret_cast<const uint4*>(router_cm + (size_t)e[q] * d);
#pragma unroll
        for (int r = 0; r < NV; ++r) w[q][r] = wp[r * kWave + lane];
    }
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        float acc = 0.0f;
#pragma unroll
        for (int r = 0; r < NV; ++r) {
            acc = dot2(xv[r].x, w[q][r].x, acc);
            acc = dot2(xv[r].y, w[q][r].y, acc);
            acc = dot2(xv[r].z, w[q][r].z, acc);
            acc = dot2(xv[r].w, w[q][r].w, acc);
        }
        out[q] = wave_allreduce_sum(acc);
    }
}

// softmax + top-k over prob[0, n_experts) and the task table of token t; called by all threads of a workgroup
// (at least 64) after the logits are in LDS.  tab / taus: LDS copies of every expert's table entry and threshold.
__device__ __forceinline__ void router_pick_and_write(const RouterArgs& a, int t, const float* prob, int* sel_id,
                                                      float* sel_w, const DevExpert* tab, const float* taus) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int slots = a.top_k + a.n_shared;
    if (a.n_experts <= 64) {
        if (wave == 0) {
            if (a.top_k > 0)
                route_select_wave64(lane < a.n_experts ? prob[lane] : 0.0f, lane, a.n_experts, a.top_k, a.renormalize,
                                    sel_id, sel_w);
            if (lane < a.n_shared) {
                sel_id[a.top_k + lane] = a.n_experts + lane;
                sel_w[a.top_k + lane] = 1.0f;
            }
        }
    } else if (tid == 0) {
        route_select(const_cast<float*>(prob), a.n_experts, a.top_k, a.n_shared, a.renormalize, sel_id, sel_w);
    }
    __syncthreads();
    // one thread per slot resolves the expert: its pointers, weight and threshold go to the task table
    if (tid < slots) {
        const int e = sel_id[tid];
        const int q = t * slots + tid;
        a.task_expert[q] = e;
        a.task_weight[q] = sel_w[tid];
        a.task_tau[q] = taus[e];
        a.task_table[q] = tab[e];
    }
}

// One workgroup of 16 waves per token.  A wave takes experts wave, wave + 16, ... and keeps kInFlight rows in flight
// at a time, so a layer with 64 experts of d <= 2048 costs one round trip to memory, not sixteen.  NV = d / 512
// pieces per lane.
template <int NV>
__global__ __launch_bounds__(1024) void router_kernel(RouterArgs a) {
    constexpr int kInFlight = NV <= 4 ? 4 : (NV <= 8 ? 2 : 1);
    __shared__ float prob[kMaxExperts];
    __shared__ int sel_id[64];
    __shared__ float sel_w[64];
    __shared__ DevExpert tab[kMaxExperts + 64];
    __shared__ float taus[kMaxExperts + 64];
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    constexpr int d = NV * 512;
    const h16* xt = a.x + (size_t)t * d;
    // every expert's table entry and threshold travel beside the router rows, so that resolving the picks costs
    // no further round trip to memory
    for (int e = tid; e < a.n_experts + a.n_shared; e += 1024) {
        tab[e] = a.table[e];
        taus[e] = a.tau[(size_t)t * a.tau_stride_t + e];
    }
    if (a.top_k > 0) {
        uint4 xv[NV];
        const uint4* xp = reinterpret_cast<const uint4*>(xt);
#pragma unroll
        for (int r = 0; r < NV; ++r) xv[r] = xp[r * kWave + lane];
        for (int e0 = wave; e0 < a.n_experts; e0 += 16 * kInFlight) {
            int e[kInFlight];
            float acc[kInFlight];
#pragma unroll
            for (int q = 0; q < kInFlight; ++q) e[q] = e0 + 16 * q < a.n_experts ? e0 + 16 * q : e0;
            router_logits<NV, kInFlight>(a.router_cm, xv, lane, e, acc);
#pragma unroll
            for (int q = 0; q < kInFlight; ++q)
                if (lane == 0 && e0 + 16 * q < a.n_experts) prob[e0 + 16 * q] = acc[q];
        }
    }
    __syncthreads();
    router_pick_and_write(a, t, prob, sel_id, sel_w, tab, taus);
}

// The same routing in two launches, for layers with many experts: one compute unit cannot pull a router matrix of a
// few hundred KB as fast as sixteen can.  The first kernel spreads the logits of a token over gridDim.x workgroups of
// four waves (a wave per expert at a time) and leaves them in a.logits[t][e]; the second picks.  The sums are formed
// exactly as in router_kernel, so both ways give the same bits.
template <int NV>
__global__ __launch_bounds__(256) void router_logits_kernel(RouterArgs a) {
    constexpr int d = NV * 512;
    constexpr int Q = NV <= 4 ? 2 : 1;
    const int t = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
    uint4 xv[NV];
    const uint4* xp = reinterpret_cast<const uint4*>(a.x + (size_t)t * d);
#pragma unroll
    for (int r = 0; r < NV; ++r) xv[r] = xp[r * kWave + lane];
    for (int e0 = gw; e0 < a.n_experts; e0 += nw * Q) {
        int e[Q];
        float acc[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) e[q] = e0 + nw * q < a.n_experts ? e0 + nw * q : e0;
        router_logits<NV, Q>(a.router_cm, xv, lane, e, acc);
#pragma unroll
        for (int q = 0; q < Q; ++q)
            if (lane == 0 && e0 + nw * q < a.n_experts) a.logits[(size_t)t * a.n_experts + e0 + nw * q] = acc[q];
    }
}

__global__ __launch_bounds__(256) void router_pick_kernel(RouterArgs a) {
    __shared__ float prob[kMaxExperts];
    __shared__ int sel_id[64];
    __shared__ float sel_w[64];
    __shared__ DevExpert tab[kMaxExperts + 64];
    __shared__ float taus[kMaxExperts + 64];
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    for (int e = tid; e < a.n_experts + a.n_shared; e += 256) {
        tab[e] = a.table[e];
        taus[e] = a.tau[(size_t)t * a.tau_stride_t + e];
        if (e < a.n_experts) prob[e] = a.logits[(size_t)t * a.n_experts + e];
    }
    __syncthreads();
    router_pick_and_write(a, t, prob, sel_id, sel_w, tab, taus);
}

hipError_t launch_router(const RouterArgs& a, int T, hipStream_t stream) {
    if (T == 0) return hipSuccess;
    const bool split = a.logits != nullptr && a.top_k > 0 && router_split_pays(a.n_experts, a.d, T);
    // workgroups per token of the split: every wave gets at least one expert, the launch about two waves of workgroups
    int per_token = (a.n_experts + 3) / 4;
    if (split) {
        const int room = 2 * num_cus() / T;
        per_token = per_token < room ? per_token : (room < 1 ? 1 : room);
    }
#define FLOE_ROUTER_NV(N)                                                                      \
    case N:                                                                                    \
        if (split) {                                                                           \
            router_logits_kernel<N><<<dim3(per_token, T), dim3(256), 0, stream>>>(a);          \
            router_pick_kernel<<<dim3(T), dim3(256), 0, stream>>>(a);                          \
        } else {                                                                               \
            router_kernel<N><<<dim3(T), dim3(1024), 0, stream>>>(a);                           \
        }                                                                                      \
        break;
    switch (a.d / 512) {
        FLOE_ROUTER_NV(1) FLOE_ROUTER_NV(2) FLOE_ROUTER_NV(3) FLOE_ROUTER_NV(4) FLOE_ROUTER_NV(5) FLOE_ROUTER_NV(6)
        FLOE_ROUTER_NV(7) FLOE_ROUTER_NV(8) FLOE_ROUTER_NV(9) FLOE_ROUTER_NV(10) FLOE_ROUTER_NV(11) FLOE_ROUTER_NV(12)
        FLOE_ROUTER_NV(13) FLOE_ROUTER_NV(14) FLOE_ROUTER_NV(15) FLOE_ROUTER_NV(16)
        default: return hipErrorInvalidValue;
    }
#undef FLOE_ROUTER_NV
    return hipGetLastError();
}

// Only the dot products, into a.logits [T][n_experts]: for a kernel behind it that does softmax and top-k itself.
hipError_t launch_router_logits(const RouterArgs& a, int T, hipStream_t stream) {
    if (T == 0 || a.n_experts == 0) return hipSuccess;
    if (!a.logits) return hipErrorInvalidValue;
    int per_token = (a.n_experts + 3) / 4;  // every wave gets at least one expert
    const int room = 2 * num_cus() / T;
    per_token = per_token < room ? per_token : (room < 1 ? 1 : room);
    switch (a.d / 512) {
#define FLOE_ROUTER_NV(N) \
    case N: router_logits_kernel<N><<<dim3(per_token, T), dim3(256), 0, stream>>>(a); break;
        FLOE_ROUTER_NV(1) FLOE_ROUTER_NV(2) FLOE_ROUTER_NV(3) FLOE_ROUTER_NV(4) FLOE_ROUTER_NV(5) FLOE_ROUTER_NV(6)
        FLOE_ROUTER_NV(7) FLOE_ROUTER_NV(8) FLOE_ROUTER_NV(9) FLOE_ROUTER_NV(10) FLOE_ROUTER_NV(11) FLOE_ROUTER_NV(12)
        FLOE_ROUTER_NV(13) FLOE_ROUTER_NV(14) FLOE_ROUTER_NV(15) FLOE_ROUTER_NV(16)
#undef FLOE_ROUTER_NV
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// one wave per task: the lanes share the per-workgroup counts of a fused launch
__global__ __launch_bounds__(256) void stats_kernel(const int32_t* task_expert, const int32_t* count, int count_parts,
                                                    const float* task_weight, SlotStat* stats, int n_tasks,
                                                    const int32_t* staged, int capacity) {
    const int q = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (q >= n_tasks) return;  // wave-uniform
    int c = 0;
    if (count_parts > 0) {
        for (int b = lane; b < count_parts; b += kWave) c += count[(size_t)q * count_parts + b];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, kWave);
    } else {
        c = count[q];
    }
    if (lane == 0) {
        SlotStat s;
        s.expert = task_expert[q];
        s.count = c;
        s.weight = task_weight[q];
        s.staged = staged ? (capacity > 0 ? min(staged[q], capacity) : staged[q]) : 0;
        stats[q] = s;
    }
}

hipError_t launch_stats(const int32_t* task_expert, const int32_t* count, int count_parts, const float* task_weight,
                        SlotStat* stats, int n_tasks, hipStream_t stream, const int32_t* staged, int capacity) {
    if (n_tasks == 0) return hipSuccess;
    stats_kernel<<<dim3((n_tasks + 3) / 4), dim3(256), 0, stream>>>(task_expert, count, count_parts, task_weight,
                                                                        stats, n_tasks, staged, capacity);
    return hipGetLastError();
}

}  // namespace floe
