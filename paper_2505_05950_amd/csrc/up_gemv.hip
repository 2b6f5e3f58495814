// S2: v = x . W_up^Q over all f channels (Alg. 1 line 2 with the quantized up projection of Sec. 3.2.2).
//
// The zero point is hoisted out of the inner loop:
//   sum_i x_i (q_i - z) s  =  s * ( sum_i x_i q_i  -  z * X_g ),   X_g = sum of x over the group,
// so the per-weight work is "extract the code, multiply-accumulate with x".
#include "floe_dev.h"
#include "launch.h"
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
template <int BITS>
__device__ __forceinline__ void load_unit(const uint32_t* __restrict__ codes, size_t unit_index, uint32_t* cw) {
    constexpr int W = PackedTraits<BITS>::kWords;
    const uint32_t* p = codes + unit_index * W;
    if (BITS == 2) {
        const uint4 q = *reinterpret_cast<const uint4*>(p);
        cw[0] = q.x; cw[1] = q.y; cw[2] = q.z; cw[3] = q.w;
    } else if (BITS == 4) {
        const uint4 q0 = reinterpret_cast<const uint4*>(p)[0], q1 = reinterpret_cast<const uint4*>(p)[1];
        cw[0] = q0.x; cw[1] = q0.y; cw[2] = q0.z; cw[3] = q0.w;
        cw[4] = q1.x; cw[5] = q1.y; cw[6] = q1.z; cw[7] = q1.w;
    } else {  // 24 bytes, 8-byte aligned
        const uint2 q0 = reinterpret_cast<const uint2*>(p)[0], q1 = reinterpret_cast<const uint2*>(p)[1],
                    q2 = reinterpret_cast<const uint2*>(p)[2];
        cw[0] = q0.x; cw[1] = q0.y; cw[2] = q1.x; cw[3] = q1.y; cw[4] = q2.x; cw[5] = q2.y;
    }
}

template <int BITS, int UPC, bool ROUTED, int kPasses, bool G32>
__global__ __launch_bounds__(256) void up_gemv_packed_kernel(TaskMap map, const h16* __restrict__ x, RouteArgs ro,
                                                             float* __restrict__ v,
                                                             const float* __restrict__ task_tau,
                                                             uint32_t* __restrict__ mask_words, int f, int gshift) {
    constexpr int CPW = kWave / UPC;  // channels per wave pass
    constexpr int d = UPC * 64;
    constexpr int kCw = PackedTraits<BITS>::kWords;
    constexpr int kWords = (kPasses * CPW * 4 + 31) / 32;  // mask words per workgroup
    static_assert((kPasses * CPW * 4) % 32 == 0, "a workgroup covers whole mask words");
    __shared__ uint32_t mw[kWords];
    __shared__ float prob[16];
    __shared__ int sel_id[16];
    __shared__ float sel_w[16];
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
    if (ROUTED) {
        // ---- S1 in place: every workgroup of the layer computes the same few dot products (n_experts <= 16,
        // the router matrix sits in L2), so no kernel of its own and no global hand-off is needed.
        // Every expert's table entry and threshold is fetched now, so that nothing has to be loaded from
        // global memory between knowing the routed expert and requesting its codes.
        if (tid < ro.n_experts + ro.n_shared) {
            tab[tid] = ro.table[tid];
            taus[tid] = ro.tau[(size_t)t * ro.tau_stride_t + tid];
        }
        // a whole wave per expert, two experts in flight per wave, fully coalesced 16-byte pieces
        constexpr int NVR = d / 512;
        uint4 xl[NVR];
        {
            const uint4* xp4 = reinterpret_cast<const uint4*>(x + (size_t)t * d);
#pragma unroll
            for (int r = 0; r < NVR; ++r) xl[r] = xp4[r * kWave + lane];
        }
        for (int e0 = wave * 2; e0 < ro.n_experts; e0 += 8) {
            uint4 w[2][NVR];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int ex = e0 + q < ro.n_experts ? e0 + q : e0;
                const uint4* wq = reinterpret_cast<const uint4*>(ro.router_cm + (size_t)ex * d);
#pragma unroll
                for (int r = 0; r < NVR; ++r) w[q][r] = wq[r * kWave + lane];
            }
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                float acc = 0.0f;
#pragma unroll
                for (int r = 0; r < NVR; ++r) {
                    acc = dot2(xl[r].x, w[q][r].x, acc);
                    acc = dot2(xl[r].y, w[q][r].y, acc);
                    acc = dot2(xl[r].z, w[q][r].z, acc);
                    acc = dot2(xl[r].w, w[q][r].w, acc);
                }
                acc = group_reduce_sum_to_last<64>(acc);
                if (lane == kWave - 1 && e0 + q < ro.n_experts) prob[e0 + q] = acc;
            }
        }
        FLOE_TL(1);
        __syncthreads();
        if (wave == 0)
            route_select_wave16(prob[lane & 15], lane, ro.n_experts, ro.top_k, ro.n_shared, ro.renormalize, sel_id, sel_w);
        __syncthreads();
        FLOE_TL(2);
        const int slot = task - t * map.slots;
        const int ex = sel_id[slot];
        e = tab[ex];
        tau = taus[ex];
        if (blockIdx.x == 0 && tid == 0) {
            ro.task_table[task] = e;
            ro.task_expert[task] = ex;
            ro.task_weight[task] = sel_w[slot];
            ro.task_tau[task] = tau;
        }
    } else {
        e = task_expert_of(map, task);
        want_mask = want_mask && task_tau != nullptr;
        if (want_mask) tau = task_tau[task];
    }

    FLOE_TL(3);
    // ---- issue the weight loads: kPasses passes of CPW channels per wave
    const int jw = (blockIdx.x * 4 + wave) * (kPasses * CPW);
    uint32_t cw[kPasses][kCw];
    uint32_t meta_s[kPasses], meta_z[kPasses];  // one fp16 (groups >= 64) or two (groups of 32) per unit
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        int j = jw + p * CPW + sub;
        j = j < f ? j : f - 1;  // keep the address in bounds; the result of a clamped lane is not stored
        load_unit<BITS>(e.codes, (size_t)j * UPC + u, cw[p]);
        if (G32) {
            const size_t mi = (size_t)j * G + 2 * u;  // even index: 4-byte aligned
            meta_s[p] = *reinterpret_cast<const uint32_t*>(e.scale + mi);
            meta_z[p] = *reinterpret_cast<const uint32_t*>(e.zero + mi);
        } else {
            const size_t mi = (size_t)j * G + ((u * 64) >> gshift);
            meta_s[p] = *reinterpret_cast<const uint16_t*>(e.scale + mi);
            meta_z[p] = *reinterpret_cast<const uint16_t*>(e.zero + mi);
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
    __syncthreads();                 // mw zeroed
    FLOE_TL(4);

#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        const int j = jw + p * CPW + sub;
        const float dot0 = half_unit_dot<BITS>(cw[p], xs, 0, magic);
        const float dot1 = half_unit_dot<BITS>(cw[p], xs, 1, magic);
        float part;
        if (G32) {
            const h16x2 s2 = as_h2(meta_s[p]), z2 = as_h2(meta_z[p]);
            part = (float)s2.x * fmaf(-(float)z2.x, Xg[0], dot0 - Xoff[0]) +
                   (float)s2.y * fmaf(-(float)z2.y, Xg[1], dot1 - Xoff[1]);
        } else {
            const float s = (float)as_h2(meta_s[p]).x, z = (float)as_h2(meta_z[p]).x;
            part = s * fmaf(-z, Xg[0] + Xg[1], (dot0 + dot1) - (Xoff[0] + Xoff[1]));
        }
        part = group_reduce_sum_to_last<UPC>(part) * inv_p;
        if (p == 0) FLOE_TL(5);
        if (u == UPC - 1 && j < f) {
            v[(size_t)task * f + j] = part;
            if (want_mask && fabsf(part) > tau) {
                const int local = j - blockIdx.x * (4 * kPasses * CPW);
                atomicOr(&mw[local >> 5], 1u << (local & 31));
            }
        }
    }
    FLOE_TL(6);
    if (want_mask) {
        __syncthreads();
        const int word = blockIdx.x * kWords + tid;
        if (tid < kWords && word < mask_words_per_task(f)) mask_words[(size_t)task * mask_words_per_task(f) + word] = mw[tid];
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

constexpr int kPassesPlain = 8, kPassesRouted = 16;

template <int BITS, int UPC>
static void launch_packed(bool routed, bool g32, int f, int n_tasks, hipStream_t stream, const TaskMap& map,
                          const h16* x, const RouteArgs& ro, float* v, const float* task_tau, uint32_t* mask_words,
                          int gshift) {
    const dim3 block(256);
    const int passes = routed ? kPassesRouted : kPassesPlain;
    const int ch_per_wg = 4 * passes * (64 / UPC);
    const dim3 grid((f + ch_per_wg - 1) / ch_per_wg, n_tasks);
    if (routed) {
        if (BITS == 2 && !g32)
            up_gemv_packed_kernel<2, UPC, true, kPassesRouted, false><<<grid, block, 0, stream>>>(map, x, ro, v, task_tau, mask_words, f, gshift);
    } else if (g32) {
        up_gemv_packed_kernel<BITS, UPC, false, kPassesPlain, true><<<grid, block, 0, stream>>>(map, x, ro, v, task_tau, mask_words, f, gshift);
    } else {
        up_gemv_packed_kernel<BITS, UPC, false, kPassesPlain, false><<<grid, block, 0, stream>>>(map, x, ro, v, task_tau, mask_words, f, gshift);
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
        case 2: up_gemv_generic_kernel<2><<<grid, block, 0, stream>>>(map, x, v, task_tau, mask_words, d, f, gshift); break;
        case 3: up_gemv_generic_kernel<3><<<grid, block, 0, stream>>>(map, x, v, task_tau, mask_words, d, f, gshift); break;
        default: up_gemv_generic_kernel<4><<<grid, block, 0, stream>>>(map, x, v, task_tau, mask_words, d, f, gshift); break;
    }
    return hipGetLastError();
}

}  // namespace floe
