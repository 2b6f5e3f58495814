// S2: v = x . W_up^Q over all f channels (Alg. 1 line 2 with the quantized up projection of Sec. 3.2.2).
//
// The zero point is hoisted out of the inner loop:
//   sum_i x_i (q_i - z) s  =  s * ( sum_i x_i q_i  -  z * X_g ),   X_g = sum of x over the group,
// so the per-weight work is "extract the code, multiply-accumulate with x".
#include "floe_dev.h"
#include "launch.h"
#include "packed_unit.h"
#include "route.h"
#include "xprep.h"

namespace floe {

// ---------------------------------------------------------------------------------------------------
// Generic kernel: any bits in {2,3,4}, any group >= 32, any d % 32 == 0 with d <= 8192.
// A lane owns "units" of 32 consecutive codes (BITS words); x sits in LDS as fp32, transposed to
// [32][U] so that the 64 lanes of a wave read consecutive addresses.
// ---------------------------------------------------------------------------------------------------
template <int BITS>
__device__ __forceinline__ uint32_t unit_code(const uint32_t (&w)[BITS], int m) {
    const int bit = m * BITS;
    const int word = bit >> 5, off = bit & 31;
    uint64_t two = w[word];
    if (off + BITS > 32) two |= (uint64_t)w[word + 1 < BITS ? word + 1 : word] << 32;
    return (uint32_t)(two >> off) & ((1u << BITS) - 1u);
}

template <int BITS>
__global__ __launch_bounds__(256) void up_gemv_generic_kernel(TaskMap map, const h16* __restrict__ x,
                                                              float* __restrict__ v,
                                                              const float* __restrict__ task_tau,
                                                              uint32_t* __restrict__ mask_words, int d, int f,
                                                              int gshift) {
    constexpr int kChPerWave = 8;
    __shared__ float xT[32 * 256];
    __shared__ float Xu[256];
    __shared__ uint32_t mw;
    const int tid = threadIdx.x;
    const int task = blockIdx.y;
    const int t = task / map.slots;
    const DevExpert e = task_expert_of(map, task);
    const int U = d >> 5;
    const h16* xt = x + (size_t)t * d;
    if (tid == 0) mw = 0u;
    for (int i = tid; i < d; i += 256) xT[(i & 31) * U + (i >> 5)] = (float)xt[i];
    __syncthreads();
    for (int u = tid; u < U; u += 256) {
        float s = 0.0f;
#pragma unroll
        for (int m = 0; m < 32; ++m) s += xT[m * U + u];
        Xu[u] = s;
    }
    __syncthreads();
    const bool want_mask = task_tau != nullptr && mask_words != nullptr;
    const float tau = want_mask ? task_tau[task] : 0.0f;
    const int wpc = d * BITS / 32;
    const int G = d >> gshift;
    const int wave = tid >> 6, lane = tid & 63;
    const int j0 = (blockIdx.x * 4 + wave) * kChPerWave;
    uint32_t bits = 0u;
    for (int c = 0; c < kChPerWave; ++c) {
        const int j = j0 + c;
        if (j >= f) break;  // wave-uniform
        float part = 0.0f;
        for (int u = lane; u < U; u += kWave) {
            const uint32_t* cw = e.codes + (size_t)j * wpc + (size_t)u * BITS;
            uint32_t w[BITS];
#pragma unroll
            for (int k = 0; k < BITS; ++k) w[k] = cw[k];
            float acc = 0.0f;
#pragma unroll
            for (int m = 0; m < 32; ++m) acc = fmaf(xT[m * U + u], (float)unit_code<BITS>(w, m), acc);
            const size_t mi = (size_t)j * G + ((u << 5) >> gshift);
            const float s = (float)e.scale[mi], z = (float)e.zero[mi];
            part = fmaf(s, fmaf(-z, Xu[u], acc), part);
        }
        part = wave_allreduce_sum(part);
        if (lane == 0) v[(size_t)task * f + j] = part;
        if (fabsf(part) > tau) bits |= 1u << (wave * kChPerWave + c);
    }
    if (want_mask) {
        if (lane == 0 && bits) atomicOr(&mw, bits);
        __syncthreads();
        if (tid == 0) mask_words[(size_t)task * mask_words_per_task(f) + blockIdx.x] = mw;
    }
}

// ---------------------------------------------------------------------------------------------------
// Packed-fp16 fast kernel: bits 2, 3 or 4; d = 64 * UPC with UPC in {16, 32, 64}; any group >= 32.
// A lane owns one 64-code unit of a channel (4 / 6 / 8 code words, loaded with 128-bit or 64-bit loads
// that the wave issues fully coalesced) and the 64 activations that meet it, prepared once per wave
// as 32 fp16 pairs (xprep.h).  A 64-lane wave therefore covers 64 / UPC channels per pass.
// Per half unit (32 codes) the lane gets sum x'q as a packed dot product, applies the group's scale and
// zero point as s * (dot - Xoff - z * Xg), and the UPC lanes of a channel are summed on the DPP path.
// Groups of 32 use one (scale, zero) per half unit, larger groups one per unit.
// All weight loads of the kPasses passes are issued before the first one is used.
// ROUTED (INT2 layer path, <= 16 experts): the workgroup first computes the router itself.
// ---------------------------------------------------------------------------------------------------
// kDepth passes of loads are in flight per wave: the next one is requested as soon as a pass has been consumed,
// so the arithmetic runs under the stream of loads instead of after it.
template <int BITS, int UPC, bool ROUTED, int kPasses, bool G32, int NW, int kDepth>
__global__ __launch_bounds__(NW * 64) void up_gemv_packed_kernel(TaskMap map, const h16* __restrict__ x, RouteArgs ro,
                                                                 float* __restrict__ v,
                                                                 const float* __restrict__ task_tau,
                                                                 uint32_t* __restrict__ mask_words, int f,
                                                                 int gshift) {
    constexpr int CPW = kWave / UPC;  // channels per wave pass
    constexpr int d = UPC * 64;
    constexpr int kCh = NW * kPasses * CPW;  // channels per workgroup
    constexpr int kWords = (kCh + 31) / 32;
    static_assert(kCh % 8 == 0, "a workgroup covers whole mask bytes");
    static_assert(kDepth >= 1 && kDepth <= kPasses, "depth of the load pipeline");
    constexpr int kParts = NW >= 16 ? 2 : 1;  // pieces a router row is cut into (one wave per piece)
    __shared__ uint32_t mw[kWords];
    __shared__ float plog[16 * kParts];
    __shared__ DevExpert tab[32];
    __shared__ float taus[32];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int sub = lane / UPC, u = lane % UPC;
    const int task = blockIdx.y;
    const int t = task / map.slots;
    const int G = d >> gshift;
    if (tid < kWords) mw[tid] = 0u;
    FLOE_TL(0);

    DevExpert e;
    float tau = 0.0f;
    bool want_mask = mask_words != nullptr;
    uint32_t raw[32];  // this lane's 64 activations
    {
        const uint4* xq = reinterpret_cast<const uint4*>(x + (size_t)t * d + u * 64);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint4 q = xq[r];
            raw[4 * r + 0] = q.x; raw[4 * r + 1] = q.y; raw[4 * r + 2] = q.z; raw[4 * r + 3] = q.w;
        }
    }
    Pick16 pick{};
    if (ROUTED) {
        // ---- S1 in place: every workgroup of the layer computes the same few dot products (n_experts <= 16,
        // the router matrix sits in L2), so no kernel of its own and no global hand-off is needed.
        // Every expert's table entry and threshold is fetched now, so that nothing has to be loaded from
        // global memory between knowing the routed expert and requesting its codes.
        if (tid < ro.n_experts + ro.n_shared) {
            tab[tid] = ro.table[tid];
            taus[tid] = ro.tau[(size_t)t * ro.tau_stride_t + tid];
        }
        route_logits_to_lds<d, NW, kParts>(x + (size_t)t * d, ro, wave, lane, plog);
        FLOE_TL(1);
        __syncthreads();
        // every wave picks the experts for itself from the logits in LDS: no second barrier, and only the ids
        // (not yet the weights) stand between the logits and the first request for codes
        float lg = 0.0f;
        if ((lane & 15) < ro.n_experts) {
#pragma unroll
            for (int q = 0; q < kParts; ++q) lg += plog[(lane & 15) * kParts + q];
        }
        const int slot = task - t * map.slots;
        int ex = ro.n_experts + (slot - ro.top_k);  // a shared expert
        if (ro.top_k > 0) {
            pick = route_pick_wave16(lg, lane, ro.n_experts, ro.top_k);
            if (slot < ro.top_k) ex = __builtin_amdgcn_readlane(pick.id, slot);
        }
        FLOE_TL(2);
        e = tab[ex];
        tau = taus[ex];
    } else {
        e = task_expert_of(map, task);
        want_mask = want_mask && task_tau != nullptr;
        if (want_mask) tau = task_tau[task];
    }

    FLOE_TL(3);
    // ---- request the first kDepth passes (a pass = CPW channels per wave)
    const int jw = (blockIdx.x * NW + wave) * (kPasses * CPW);
    UnitLoad<BITS, UPC, G32> ld[kDepth];
    auto channel_of = [&](int p) {
        const int j = jw + p * CPW + sub;
        return j < f ? j : f - 1;  // keep the address in bounds; the result of a clamped lane is not stored
    };
#pragma unroll
    for (int p = 0; p < kDepth; ++p) ld[p].issue(e, channel_of(p), u, G, gshift);
    FLOE_TL(7);

    if (ROUTED && blockIdx.x == 0 && wave == 0) {  // the task's routing record, for the kernels that follow
        const int slot = task - t * map.slots;
        float wgt = 1.0f;
        if (ro.top_k > 0) {
            const float wl = route_weight_wave16(pick, ro.top_k, ro.renormalize);
            if (slot < ro.top_k) wgt = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wl), slot));
        }
        if (lane == 0) {
            const int ex = slot < ro.top_k ? __builtin_amdgcn_readlane(pick.id, slot) : ro.n_experts + (slot - ro.top_k);
            ro.task_table[task] = e;
            ro.task_expert[task] = ex;
            ro.task_weight[task] = wgt;
            ro.task_tau[task] = tau;
        }
    }

    // ---- activations of this lane's unit: 32 scaled fp16 pairs
    uint32_t xs[32];
    float Xg[2], Xoff[2];
    // every group of UPC lanes holds the whole token, so the wave-wide maximum is the token's
    const float amax = wave_allreduce_max_nonneg(unit_amax(raw));
    const int down = xprep_down<BITS>(amax);
    const float inv_p = ldexpf(1.0f, down);
    unit_prepare<BITS>(raw, down, xs, Xoff, Xg);
    uint32_t magic = 0x3C003C00u;
    asm volatile("" : "+v"(magic));  // keep it in a VGPR: v_and_or_b32 takes one scalar operand only
    FLOE_TL(8);
    if (!ROUTED) __syncthreads();  // mw zeroed (the routed path has passed a barrier already)
    FLOE_TL(4);

#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        const int j = jw + p * CPW + sub;
        UnitLoad<BITS, UPC, G32>& L = ld[p % kDepth];
        float part = unit_value<BITS, UPC, G32>(L, xs, Xoff, Xg, magic);
        if (p + kDepth < kPasses) L.issue(e, channel_of(p + kDepth), u, G, gshift);
        part = group_reduce_sum_to_last<UPC>(part) * inv_p;
        if (p == 0) FLOE_TL(5);
        if (u == UPC - 1 && j < f) {
            v[(size_t)task * f + j] = part;
            if (want_mask && fabsf(part) > tau) {
                const int local = j - blockIdx.x * kCh;
                atomicOr(&mw[local >> 5], 1u << (local & 31));
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the request for pass p + kDepth where it is
    }
    FLOE_TL(6);
    if (want_mask) {
        // the workgroup's channels start on a byte of the task's mask; the last workgroup also clears what is
        // left of the last word, so that every byte of the mask is written by exactly one workgroup
        __syncthreads();
        const int n_bytes = mask_words_per_task(f) * 4;
        uint8_t* mb = reinterpret_cast<uint8_t*>(mask_words + (size_t)task * mask_words_per_task(f));
        const int b = blockIdx.x * (kCh / 8) + tid;
        const bool last = blockIdx.x == gridDim.x - 1;
        if (tid < kCh / 8) {
            if (b < n_bytes) mb[b] = reinterpret_cast<const uint8_t*>(mw)[tid];
        } else if (last && tid < kCh / 8 + 4 && b < n_bytes) {
            mb[b] = 0;
        }
    }
}

#ifdef FLOE_TIMELINE
extern "C" int floe_debug_set_timeline_up_gemv(unsigned long long* p) {
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_timeline), &p, sizeof(p));
}
#endif

static int ilog2_exact(int g) {
    int s = 0;
    while ((1 << s) < g) ++s;
    return s;
}

// Launch shapes.  Plain: 4 waves x 8 passes.  Routed (the T-small layer path): 16 waves x 7 passes, which at
// d = 4096, f = 14336 and two tasks is exactly one workgroup per compute unit (2 x 128 workgroups of 112 channels).
constexpr int kPassesPlain = 8, kWavesPlain = 4;
#ifndef FLOE_RW
#define FLOE_RW 8
#define FLOE_RP 14
#define FLOE_RD 6
#endif
constexpr int kPassesRouted = FLOE_RP, kWavesRouted = FLOE_RW, kDepthRouted = FLOE_RD;
constexpr int kDepthPlain = 4;

template <int BITS, int UPC>
static void launch_packed(bool routed, bool g32, int f, int n_tasks, hipStream_t stream, const TaskMap& map,
                          const h16* x, const RouteArgs& ro, float* v, const float* task_tau, uint32_t* mask_words,
                          int gshift) {
    const int waves = routed ? kWavesRouted : kWavesPlain;
    const int passes = routed ? kPassesRouted : kPassesPlain;
    const dim3 block(waves * 64);
    const int ch_per_wg = waves * passes * (64 / UPC);
    const dim3 grid((f + ch_per_wg - 1) / ch_per_wg, n_tasks);
    if (routed) {
        if (BITS == 2 && !g32)
            up_gemv_packed_kernel<2, UPC, true, kPassesRouted, false, kWavesRouted, kDepthRouted><<<grid, block, 0, stream>>>(map, x, ro, v, task_tau, mask_words, f, gshift);
    } else if (g32) {
        up_gemv_packed_kernel<BITS, UPC, false, kPassesPlain, true, kWavesPlain, kDepthPlain><<<grid, block, 0, stream>>>(map, x, ro, v, task_tau, mask_words, f, gshift);
    } else {
        up_gemv_packed_kernel<BITS, UPC, false, kPassesPlain, false, kWavesPlain, kDepthPlain><<<grid, block, 0, stream>>>(map, x, ro, v, task_tau, mask_words, f, gshift);
    }
}

template <int BITS>
static void launch_packed_upc(int upc, bool routed, bool g32, int f, int n_tasks, hipStream_t stream, const TaskMap& map,
                              const h16* x, const RouteArgs& ro, float* v, const float* task_tau, uint32_t* mask_words,
                              int gshift) {
    if (upc == 64) launch_packed<BITS, 64>(routed, g32, f, n_tasks, stream, map, x, ro, v, task_tau, mask_words, gshift);
    else if (upc == 32) launch_packed<BITS, 32>(routed, g32, f, n_tasks, stream, map, x, ro, v, task_tau, mask_words, gshift);
    else launch_packed<BITS, 16>(routed, g32, f, n_tasks, stream, map, x, ro, v, task_tau, mask_words, gshift);
}

hipError_t launch_up_gemv(const TaskMap& map, const h16* x, const RouteArgs* route, float* v, const float* task_tau,
                          uint32_t* mask_words, int d, int f, int bits, int group, int n_tasks, hipStream_t stream) {
    if (f == 0 || n_tasks == 0) return hipSuccess;
    const int gshift = ilog2_exact(group);
    dim3 block(256);
    if (packed_fast_shape(d, bits, group)) {
        const int upc = d / 64;
        const bool routed = route != nullptr;
        const bool g32 = group == 32;
        if (routed && !(bits == 2 && !g32)) return hipErrorInvalidValue;
        RouteArgs ro{};
        if (routed) ro = *route;
        if (bits == 2) launch_packed_upc<2>(upc, routed, g32, f, n_tasks, stream, map, x, ro, v, task_tau, mask_words, gshift);
        else if (bits == 3) launch_packed_upc<3>(upc, false, g32, f, n_tasks, stream, map, x, ro, v, task_tau, mask_words, gshift);
        else launch_packed_upc<4>(upc, false, g32, f, n_tasks, stream, map, x, ro, v, task_tau, mask_words, gshift);
        return hipGetLastError();
    }
    if (route != nullptr) return hipErrorInvalidValue;  // in-place routing exists only in the packed INT2 kernel
    dim3 grid((f + 31) / 32, n_tasks);
    switch (bits) {
        case 1: up_gemv_generic_kernel<1><<<grid, block, 0, stream>>>(map, x, v, task_tau, mask_words, d, f, gshift); break;
        case 8: up_gemv_generic_kernel<8><<<grid, block, 0, stream>>>(map, x, v, task_tau, mask_words, d, f, gshift); break;
        case 2: up_gemv_generic_kernel<2><<<grid, block, 0, stream>>>(map, x, v, task_tau, mask_words, d, f, gshift); break;
        case 3: up_gemv_generic_kernel<3><<<grid, block, 0, stream>>>(map, x, v, task_tau, mask_words, d, f, gshift); break;
        default: up_gemv_generic_kernel<4><<<grid, block, 0, stream>>>(map, x, v, task_tau, mask_words, d, f, gshift); break;
    }
    return hipGetLastError();
}

}  // namespace floe
