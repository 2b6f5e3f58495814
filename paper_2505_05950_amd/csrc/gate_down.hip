// S3 (compaction) + S4 + S5: gathered gate GEMV with fused SiLU and the product with v, then the gathered
// down GEMV (Alg. 1 lines 3-5), reading only the compact [gate | down] chunks (Sec. 3.4.2) of the
// selected channels.
//
// Everything here is bound by memory latency, not arithmetic (a Mixtral-shaped expert at 90 % sparsity
// leaves about 11 channels of 16 KiB per compute unit), so the kernel is organised around ONE round
// trip to HBM per batch of channels:
//   * a workgroup takes a contiguous slice [k0, k1) of the task's ascending channel list.  With
//     FROM_MASK the list is never materialised by a kernel of its own: the GEMV kernel left one mask
//     bit per channel, every workgroup prefix-sums the popcounts of the task's mask words in LDS and
//     finds its own channels by binary search (and writes them to idx for the callers that want the list);
//   * for a batch of B channels every load is issued before anything is used: wave w requests the whole
//     gate columns of channels w, w+4, ... and every thread requests its 16-byte pieces of all B down rows;
//   * gate: x . column by packed dot products and a DPP wave reduction, h = SiLU(g) * v_j * scale -> LDS;
//   * down: the four waves split the d output columns between them, so a thread adds h_c * (its pieces)
//     into 8 fp32 accumulators per piece and no reduction between waves is needed;
//   * the workgroup stores one partial y; S6 adds the partials of all workgroups and slots.
#include "floe_dev.h"
#include "launch.h"

namespace floe {

constexpr int kMaxMaskWords = 2048;  // FROM_MASK handles f <= 65536

template <int NV>
struct GdTile {
    static constexpr int BG = NV >= 24 ? 1 : (24 / NV > 4 ? 4 : (24 / NV < 1 ? 1 : 24 / NV));  // gate channels per wave
    static constexpr int B = 4 * BG;                                                          // channels per batch
    static constexpr int VPR = 64 * NV;                 // uint4 per gate column / down row (d / 8)
    static constexpr int RG = (VPR + 255) / 256;        // down pieces per thread per channel
};

template <int NV, bool FROM_MASK, bool HAS_ROWS = false>  // d = 512 * NV
__global__ __launch_bounds__(256) void gate_down_kernel(TaskMap map, const h16* __restrict__ staged_base, int gd_rows,
                                                        const h16* __restrict__ x, const float* __restrict__ v,
                                                        const uint32_t* __restrict__ mask_words,
                                                        int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                        const float* __restrict__ task_scale,
                                                        float* __restrict__ partial, int f,
                                                        const int32_t* __restrict__ rows,
                                                        const int32_t* __restrict__ order) {
    constexpr int d = 512 * NV;
    using Tile = GdTile<NV>;
    constexpr int BG = Tile::BG, B = Tile::B, VPR = Tile::VPR, RG = Tile::RG;
    __shared__ int prefix[FROM_MASK ? kMaxMaskWords + 1 : 1];
    __shared__ uint32_t words[FROM_MASK ? kMaxMaskWords : 1];
    __shared__ int wave_tot[4];
    __shared__ int jl[256];
    __shared__ float hl[B];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    // order (batches): row y of the grid works on task order[y]; the tasks are sorted by expert, so the workgroups that
    // run at the same time belong to few experts, and with a block count that is a multiple of the number of XCDs the
    // workgroups of one channel range sit on one XCD: a row that several tokens selected is fetched from HBM once and
    // served to the others by that XCD's L2
    const int task = order ? order[blockIdx.y] : blockIdx.y;
    const int t = task / map.slots;
    const DevExpert e = task_expert_of(map, task);
    const float out_scale = task_scale ? task_scale[task] : 1.0f;
    const float* vt = v + (size_t)task * f;
    // staged: the task's selected chunks sit in rows 0..K-1 of its own slab of the staging buffer
    const bool staged = staged_base != nullptr;
    // rows (staged only): row of the staging buffer that holds the k-th channel of the task's list, -1 = absent
    const h16* gdp = staged ? (HAS_ROWS ? staged_base : staged_base + (size_t)task * gd_rows * 2 * d) : e.gd;
    const int32_t* rw = HAS_ROWS ? rows + (size_t)task * f : nullptr;

    FLOE_TL(0);
    uint4 xr[NV];
    {
        const uint4* xp = reinterpret_cast<const uint4*>(x + (size_t)t * d);
#pragma unroll
        for (int r = 0; r < NV; ++r) xr[r] = xp[r * kWave + lane];
    }

    // ---- how many channels, and which slice is ours
    int K;
    if (FROM_MASK) {
        const int nwords = mask_words_per_task(f);
        const int wpt = (nwords + 255) / 256;  // consecutive words per thread (<= 8)
        const uint32_t* mw = mask_words + (size_t)task * nwords;
        uint32_t my[8];
        int mine = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int w = tid * wpt + i;
            my[i] = (i < wpt && w < nwords) ? mw[w] : 0u;
            mine += __popc(my[i]);
        }
        // inclusive scan over the wave, then over the four waves
        int inc = mine;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int up = __shfl_up(inc, o, kWave);
            if (lane >= o) inc += up;
        }
        if (lane == kWave - 1) wave_tot[wave] = inc;
        __syncthreads();
        int base = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) base += w < wave ? wave_tot[w] : 0;
        K = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
        int run = base + inc - mine;  // exclusive prefix of this thread's first word
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int w = tid * wpt + i;
            if (i < wpt && w < nwords) {
                prefix[w] = run;
                words[w] = my[i];
                run += __popc(my[i]);
            }
        }
        if (tid == 0) {
            prefix[nwords] = K;
            if (count && blockIdx.x == 0) count[task] = K;
        }
        __syncthreads();
    } else {
        K = count[task];
    }
    FLOE_TL(1);
    const int Kc = min(K, (staged && !HAS_ROWS) ? gd_rows : f);
    const int per = (Kc + (int)gridDim.x - 1) / (int)gridDim.x;
    const int k0 = min(Kc, (int)blockIdx.x * per);
    const int k1 = min(Kc, k0 + per);

    float acc[RG * 8];
#pragma unroll
    for (int i = 0; i < RG * 8; ++i) acc[i] = 0.0f;

    for (int kc = k0; kc < k1; kc += 256) {
        const int n = min(256, k1 - kc);
        if (tid < n) {
            const int k = kc + tid;
            int j;
            if (FROM_MASK) {
                int lo = 0, hi = mask_words_per_task(f);
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (prefix[mid] <= k) lo = mid; else hi = mid;
                }
                uint32_t wbits = words[lo];
                for (int r = k - prefix[lo]; r > 0; --r) wbits &= wbits - 1;  // drop the r lowest set bits
                j = lo * 32 + (__ffs(wbits) - 1);
                if (idx) idx[(size_t)task * f + k] = j;
            } else {
                j = idx[(size_t)task * f + k];
                if ((unsigned)j >= (unsigned)f) j = -1;  // a caller-supplied list may hold junk: never leave the matrix
            }
            jl[tid] = j;
        }
        __syncthreads();
        FLOE_TL(2);

        for (int b0 = 0; b0 < n; b0 += B) {
            // ---- all loads of the batch
            uint4 gv[BG][NV];
            uint4 dv[B][RG];
            float vj[BG];
#pragma unroll
            for (int i = 0; i < BG; ++i) {
                const int c = b0 + wave + 4 * i;
                int j = c < n ? jl[c] : -1;
                vj[i] = j >= 0 ? vt[j] : 0.0f;  // same address in every lane; needed only after the dot product
                size_t row;
                if (HAS_ROWS) {
                    const int rr = j >= 0 ? rw[kc + c] : -1;
                    if (rr < 0) j = -1;  // the chunk is not in the staging buffer (overflow): the channel is left out
                    row = (size_t)(rr < 0 ? 0 : rr);
                } else {
                    row = staged ? (size_t)(kc + c) : (size_t)(j < 0 ? 0 : j);
                }
                const uint4* gp = reinterpret_cast<const uint4*>(gdp + row * 2 * d);
#pragma unroll
                for (int r = 0; r < NV; ++r) gv[i][r] = j >= 0 ? gp[r * kWave + lane] : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int cc = 0; cc < B; ++cc) {
                const int c = b0 + cc;
                int j = c < n ? jl[c] : -1;
                size_t row;
                if (HAS_ROWS) {
                    const int rr = j >= 0 ? rw[kc + c] : -1;
                    if (rr < 0) j = -1;
                    row = (size_t)(rr < 0 ? 0 : rr);
                } else {
                    row = staged ? (size_t)(kc + c) : (size_t)(j < 0 ? 0 : j);
                }
                const uint4* dp = reinterpret_cast<const uint4*>(gdp + row * 2 * d + d);
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    const int piece = tid + 256 * r;
                    dv[cc][r] = (j >= 0 && piece < VPR) ? dp[piece] : make_uint4(0u, 0u, 0u, 0u);
                }
            }
            FLOE_TL(3);
            // ---- gate: h_c = SiLU(x . gate_c) * v_c * scale
#pragma unroll
            for (int i = 0; i < BG; ++i) {
                const int c = b0 + wave + 4 * i;
                float g = 0.0f;
#pragma unroll
                for (int r = 0; r < NV; ++r) {
                    g = dot2(xr[r].x, gv[i][r].x, g);
                    g = dot2(xr[r].y, gv[i][r].y, g);
                    g = dot2(xr[r].z, gv[i][r].z, g);
                    g = dot2(xr[r].w, gv[i][r].w, g);
                }
                g = wave_allreduce_sum(g);
                bool present = c < n && jl[c] >= 0;
                if (HAS_ROWS) present = present && rw[kc + c] >= 0;
                if (lane == 0) hl[wave + 4 * i] = present ? silu(g) * vj[i] * out_scale : 0.0f;
            }
            FLOE_TL(4);
            __syncthreads();
            FLOE_TL(5);
            // ---- down: acc += h_c * (this thread's pieces of row c)
#pragma unroll
            for (int cc = 0; cc < B; ++cc) {
                const float h = hl[cc];
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    const uint32_t wds[4] = {dv[cc][r].x, dv[cc][r].y, dv[cc][r].z, dv[cc][r].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const h16x2 p = as_h2(wds[q]);
                        acc[r * 8 + 2 * q + 0] = fmaf(h, (float)p.x, acc[r * 8 + 2 * q + 0]);
                        acc[r * 8 + 2 * q + 1] = fmaf(h, (float)p.y, acc[r * 8 + 2 * q + 1]);
                    }
                }
            }
            FLOE_TL(6);
            __syncthreads();  // hl is rewritten by the next batch
        }
        __syncthreads();  // jl is rewritten by the next chunk
    }

    // thread owns output columns [8 * piece, 8 * piece + 8) for piece = tid + 256 r
    float* out = partial + ((size_t)task * gridDim.x + blockIdx.x) * d;
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const int piece = tid + 256 * r;
        if (piece < VPR) {
            float4* o4 = reinterpret_cast<float4*>(out + (size_t)piece * 8);
            o4[0] = make_float4(acc[r * 8 + 0], acc[r * 8 + 1], acc[r * 8 + 2], acc[r * 8 + 3]);
            o4[1] = make_float4(acc[r * 8 + 4], acc[r * 8 + 5], acc[r * 8 + 6], acc[r * 8 + 7]);
        }
    }
    FLOE_TL(7);
}

#ifdef FLOE_TIMELINE
extern "C" int floe_debug_set_timeline_gate_down(unsigned long long* p) {
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_timeline), &p, sizeof(p));
}
#endif

int gd_blocks(int n_tasks, int f) {
    if (n_tasks <= 0) return 1;
    int nblk = num_cus() / n_tasks;
    nblk = nblk < 1 ? 1 : nblk;
    // batches: a multiple of the 8 XCDs, so that block b of every task runs on
    // XCD b % 8 (workgroups go to the XCDs in turn) and tasks that share an expert share its rows in that XCD's L2
    if (n_tasks > kExpertOrderTasks) nblk = (nblk + 7) / 8 * 8;
    const int by_f = (f + 3) / 4;  // a workgroup should have at least a few channels to look at
    nblk = nblk > by_f ? by_f : nblk;
    return nblk < 1 ? 1 : nblk;
}

template <int NV>
static hipError_t launch_nv(const TaskMap& map, const h16* staged, int gd_rows, const h16* x, const float* v,
                            const uint32_t* mask_words, int32_t* idx, int32_t* count, const float* task_scale,
                            float* partial, int f, int n_tasks, int nblk, const int32_t* rows, const int32_t* order,
                            hipStream_t stream) {
    dim3 grid(nblk, n_tasks), block(256);
    if (mask_words)
        gate_down_kernel<NV, true><<<grid, block, 0, stream>>>(map, staged, gd_rows, x, v, mask_words, idx, count,
                                                              task_scale, partial, f, nullptr, order);
    else if (rows)
        gate_down_kernel<NV, false, true><<<grid, block, 0, stream>>>(map, staged, gd_rows, x, v, nullptr, idx, count,
                                                                     task_scale, partial, f, rows, order);
    else
        gate_down_kernel<NV, false><<<grid, block, 0, stream>>>(map, staged, gd_rows, x, v, nullptr, idx, count,
                                                               task_scale, partial, f, nullptr, order);
    return hipGetLastError();
}

hipError_t launch_gate_down(const TaskMap& map, const h16* staged, int gd_rows, const h16* x, const float* v,
                            const uint32_t* mask_words, int32_t* idx, int32_t* count, const float* task_scale,
                            float* partial, int d, int f, int n_tasks, int nblk, hipStream_t stream,
                            const int32_t* rows, const int32_t* order) {
    if (n_tasks == 0) return hipSuccess;
    if (rows && (mask_words || !staged)) return hipErrorInvalidValue;  // explicit rows go with a staged list
    if (mask_words && mask_words_per_task(f) > kMaxMaskWords) return hipErrorInvalidValue;
#define FLOE_NV_CASE(N)                                                                                            \
    case N:                                                                                                        \
        return launch_nv<N>(map, staged, gd_rows, x, v, mask_words, idx, count, task_scale, partial, f, n_tasks, nblk, \
                            rows, order, stream);
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
// A workgroup owns 32 output columns of one token: 8 threads (one float4 each) cover the columns,
// the 32 thread rows split the partials between them (eight loads in flight each); the sums meet by lane
// exchange inside a wave and in LDS across the four waves (a fixed order, so the result is reproducible).
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ partial, int d, int per_token,
                                                      float* __restrict__ y_acc, h16* __restrict__ y_half) {
    __shared__ float4 red[4][8];
    const int t = blockIdx.y;
    const int cg = threadIdx.x & 7, pg = threadIdx.x >> 3;
    const int c4 = blockIdx.x * 8 + cg;  // column / 4   (d % 32 == 0)
    const float4* p = reinterpret_cast<const float4*>(partial + (size_t)t * per_token * d) + c4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int b0 = pg; b0 < per_token; b0 += 32 * 8) {
        float4 a[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {  // eight independent loads in flight
            const int b = b0 + 32 * i;
            a[i] = b < per_token ? p[(size_t)b * (d / 4)] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) { s.x += a[i].x; s.y += a[i].y; s.z += a[i].z; s.w += a[i].w; }
    }
    // the eight thread rows of a wave meet by lane exchange (lane = row * 8 + column group), the four waves in LDS
#pragma unroll
    for (int o = 8; o < 64; o <<= 1) {
        s.x += __shfl_xor(s.x, o, kWave);
        s.y += __shfl_xor(s.y, o, kWave);
        s.z += __shfl_xor(s.z, o, kWave);
        s.w += __shfl_xor(s.w, o, kWave);
    }
    if ((pg & 7) == 0) red[pg >> 3][cg] = s;
    __syncthreads();
    if (pg != 0) return;
#pragma unroll
    for (int r = 1; r < 4; ++r) {
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
    dim3 grid(d / 32, T);
    combine_kernel<<<grid, dim3(256), 0, stream>>>(partial, d, slots * nblk, y_acc, y_half);
    return hipGetLastError();
}

}  // namespace floe
