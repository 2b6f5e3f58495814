// (S1 +) S2-S5 of a small decode batch in ONE kernel (Sec. 3.3 router; Alg. 1 steps 2-5 with the quantized up
// projection of Sec. 3.2.2 and the compact [gate | down] chunks of Sec. 3.4.2).  Template for every bit width;
// instantiated in fused_int2.hip / fused_int3.hip / fused_int4.hip.
//
// Why one kernel: the threshold test of Alg. 1 is per channel, so a workgroup that has computed v for a block
// of channels knows, without hearing from anybody else, which of ITS channels take part in steps 4-5; it can
// run them itself and hand over a partial y.  v, the mask and the index list never leave the compute unit, and
// two kernel boundaries (launch, drain, dependent prologue) disappear.
//
// Why two kinds of waves: a layer-token moves 37 MB of codes and 47 MB of selected chunks, and the kernel lasts
// as long as that stream plus whatever is not overlapped with it.  The chunk of a selected channel should
// therefore be requested the moment the channel is known, while the code stream keeps flowing.  The hardware
// counts a wave's outstanding loads in order, so a wave that mixes a deep static pipeline of code loads with
// data-dependent chunk loads ends up waiting for one because of the other.  So the workgroup (12 waves) splits:
//   * 4 producer waves stream the codes (kDepth passes in flight each), compute v_j on packed fp16 dot
//     products (see up_gemv.hip / xprep.h), compare with tau and push (j, v_j * routing weight) of every
//     selected channel into a queue in LDS - one queue per producer, written by nobody else;
//   * 8 consumer waves, two per queue taking its entries in turn: request the chunk (a whole gate column and down row per
//     wave, coalesced), x . gate on dot2 + DPP, SiLU, and h * down row into d/64 fp32 accumulators per lane.
// A producer never waits for a consumer; a consumer polls its queue in LDS and leaves once its producer has
// raised its flag and the queue is empty, so every wave reaches the final barrier.  Queue k of workgroup b
// always holds the same channels in the same order, hence the sums are formed in a fixed order and the result
// is reproducible bit for bit.  After the barrier the four accumulators meet in LDS and the workgroup stores
// one partial y; S6 (combine_kernel) adds the partials.
#pragma once

#include "floe_dev.h"
#include "launch.h"
#include "packed_unit.h"
#include "route.h"
#include "xprep.h"

namespace floe {

constexpr int kFusedProducers = fused_producers;
constexpr int kFusedCpp = 2;                                    // consumer waves per producer (queue entries dealt in turn)
constexpr int kFusedConsumers = kFusedProducers * kFusedCpp;
constexpr int kFusedThreads = (kFusedProducers + kFusedConsumers) * 64;

// Queue words are read and written with volatile accesses that are typed as LDS: a volatile access through a generic
// pointer becomes a FLAT instruction with system scope, which ticks the vector-memory counter as well and makes the
// producer wait for its code loads whenever it pushes an entry.
#define FLOE_LDS __attribute__((address_space(3)))
__device__ __forceinline__ int lds_peek(const int* p) { return *(const volatile FLOE_LDS int*)p; }
__device__ __forceinline__ void lds_poke(int* p, int v) { *(volatile FLOE_LDS int*)p = v; }
__device__ __forceinline__ void lds_poke(float* p, float v) { *(volatile FLOE_LDS float*)p = v; }

// Codes that go from memory straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes land at base + 16 l, no
// register is held while the load is in flight, so a wave can keep many more passes on their way).  The compiler
// knows no finer rule for such a load than "wait for all of them before any LDS read that may touch the same
// array", which would serialise the pipeline; the read-back is therefore issued here by hand, after a wait that
// names how many younger vector-memory operations may still be outstanding.
template <int N>
__device__ __forceinline__ void wait_vm_all_but() {  // s_waitcnt vmcnt(N) only (gfx9 encoding: bits 3:0 and 15:14)
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// A lane's unit of 64 codes travels in kPieces loads of 16 bytes; piece k of all 64 lanes lands contiguously at
// slot + k * 1024.  kPieces = 0: the width keeps its codes in registers.  Only INT2 is staged: INT4 (two pieces per
// unit) measured slower that way (16.8 against 15.9 us per expert at 90 %), INT3 units are 24 bytes, 8-byte aligned.
template <int BITS> struct StageTraits;
template <> struct StageTraits<2> { static constexpr int kPieces = 1, kPieceBytes = 16; };
template <> struct StageTraits<3> { static constexpr int kPieces = 0, kPieceBytes = 16; };
template <> struct StageTraits<4> { static constexpr int kPieces = 0, kPieceBytes = 16; };
template <int BITS> constexpr int stage_slot_bytes() { return StageTraits<BITS>::kPieces * StageTraits<BITS>::kPieceBytes * 64; }
template <int BITS> constexpr bool staged_codes() { return StageTraits<BITS>::kPieces > 0; }

__device__ __forceinline__ void dma16_to_lds(const void* src, void* lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const FLOE_GLOBAL void*)src, (FLOE_LDS void*)lds_wave_base, 16, 0, 0);
}
// Read a lane's piece back.  The compiler does not know that this LDS read exists (it would make it wait for every
// direct-to-LDS load), so request and arrival are two statements, one pass apart: nothing may touch the registers
// between them, which the second statement enforces by taking them as in/out operands.
__device__ __forceinline__ void lds_piece_request(const void* lds_ptr, u32x4& q) {
    const uint32_t a = (uint32_t)(uintptr_t)(const FLOE_LDS void*)lds_ptr;
    asm volatile("ds_read_b128 %0, %1" : "=v"(q) : "v"(a) : "memory");
}
__device__ __forceinline__ void lds_piece_arrived(u32x4& q) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(q) : : "memory"); }

// ROUTED: 2 = the workgroup routes in place (<= 16 experts), 1 = it picks in place on logits formed by a kernel in front
// (<= 64 experts), 0 = the task's expert comes from `map`, its
// threshold from task_tau and its output scale from task_scale (nullptr = 1).
// n_pass channels-per-wave passes per producer (at most kPasses, which sizes the queues), kDepth of them in flight; with
// codes staged through LDS n_pass is a multiple of kDepth.  v_out (optional): v[task][f].
template <int BITS, int UPC, bool G32, int ROUTED, int kPasses, int kDepth>
__global__ __launch_bounds__(kFusedThreads, fused_wgs_per_cu) void fused_ffn_kernel(TaskMap map, const h16* __restrict__ x, RouteArgs ro,
                                                                  const float* __restrict__ task_tau,
                                                                  const float* __restrict__ task_scale, int f,
                                                                  int n_pass_arg, int gshift, float* __restrict__ v_out,
                                                                  float* __restrict__ partial,
                                                                  int32_t* __restrict__ wg_count) {
    constexpr int d = 64 * UPC;
    constexpr int CPW = kWave / UPC;      // channels per wave pass
    constexpr int NV = d / 512;           // uint4 per lane of a gate column / down row
    constexpr int kQ = kPasses * CPW;     // queue capacity
    // the small size runs exactly kPasses passes, the large one what the launch says
    const int n_pass = kPasses == kFusedMaxPasses ? n_pass_arg : kPasses;
    const int nq = n_pass * CPW;          // channels per producer = the most a queue can receive
    static_assert(kDepth >= 1 && kDepth <= kPasses, "depth of the load pipeline");
    __shared__ float plog[32];                  // router: two partial dot products per expert
    __shared__ DevExpert tab[kFusedMaxRouted + 16];
    __shared__ float taus[kFusedMaxRouted + 16];
    __shared__ int qj[kFusedProducers][kQ];     // selected channel, -1 = not written yet
    __shared__ float qh[kFusedProducers][kQ];   // its v times the routing weight
    __shared__ int done[kFusedProducers];
    __shared__ int expert_of_queue[kFusedProducers];  // the expert its producer picked (-1 = not yet), for the consumers
    __shared__ int n_sel;
    __shared__ float yred[kFusedConsumers][d];
    __shared__ uint4 xlds[d / 8];               // the token, for the consumers' gate dot products
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;  // the wave index as a scalar
    // Which (task, channel block) this workgroup takes.  Workgroups go to the eight XCDs round-robin in launch order.
    // With several tasks and a block count that is a multiple of eight, the tasks' workgroups for one channel block are
    // launched next to each other on one XCD: tasks that were routed to the same expert then read that block's codes
    // (and the rows both select) from HBM once, the later ones from the L2.
    int task = blockIdx.y, blk = blockIdx.x;
    if (gridDim.y > 1 && (gridDim.x & 7) == 0) {
        const int L = blockIdx.y * gridDim.x + blockIdx.x, s_ = L >> 3;
        task = s_ % (int)gridDim.y;
        blk = 8 * (s_ / (int)gridDim.y) + (L & 7);
    }
    const int t = task / map.slots;
    const int slot = task - t * map.slots;
    const h16* xt = x + (size_t)t * d;
#pragma unroll
    for (int w = 0; w < kFusedProducers; ++w)
        for (int i = tid; i < nq; i += kFusedThreads) qj[w][i] = -1;
    if (tid < kFusedProducers) {
        done[tid] = 0;
        expert_of_queue[tid] = -1;
    }
    if (tid == 0) n_sel = 0;
    for (int i = tid; i < d / 8; i += kFusedThreads) xlds[i] = reinterpret_cast<const uint4*>(xt)[i];
    FLOE_TL(0);

    const bool producer = wave < kFusedProducers;
    const int u = lane % UPC, sub = CPW == 1 ? 0 : lane / UPC;
    DevExpert e{};
    float tau = 0.0f;
    Pick16 pick{};
    int ex = 0;
    if (ROUTED) {
        // ---- S1 in place.  Every workgroup of the launch repeats it, so its cost is the length of the prologue of all of
        // them: the router rows are requested first (half a row per item, dealt over all waves), the token comes from the copy in
        // LDS once the barrier has passed (read from memory by every wave it doubled the bytes a workgroup pulls through
        // the L2), and only the producers work out the pick: they need it to request codes, while a consumer needs
        // the expert's gate/down address no earlier than its first queue entry and would only take issue slots from the
        // two producers on its SIMD.
        if (tid < ro.n_experts + ro.n_shared) {
            tab[tid] = ro.table[tid];
            taus[tid] = ro.tau[(size_t)t * ro.tau_stride_t + tid];
        }
        float lg = 0.0f;  // producers: the logit of the expert this lane stands for
        if constexpr (ROUTED == 1) {
            // the dot products were formed by a kernel in front (more than 16 experts: a workgroup that repeated them
            // would pull the whole router matrix through its L2 port); lane e holds expert e
            if (producer && lane < ro.n_experts) lg = ro.logits[(size_t)t * ro.n_experts + lane];
            __syncthreads();  // xlds, queues, flags and the table are set up
        } else {
            constexpr int kParts = 2, NVR = d / 512 / kParts;
            constexpr int NW = kFusedThreads / 64;
            constexpr int kItems = (16 * kParts + NW - 1) / NW;  // items a wave may have to take (<= 16 experts)
            const int n_items = ro.n_experts * kParts;
            uint4 rw[kItems][NVR];
#pragma unroll
            for (int q = 0; q < kItems; ++q) {
                const int it = wave + q * NW;
                if (it >= n_items) break;  // wave-uniform
                const uint4* wq = reinterpret_cast<const uint4*>(ro.router_cm + (size_t)(it / kParts) * d);
#pragma unroll
                for (int r = 0; r < NVR; ++r) rw[q][r] = wq[((it % kParts) * NVR + r) * kWave + lane];
            }
            __syncthreads();  // xlds, queues and flags are set up
#pragma unroll
            for (int q = 0; q < kItems; ++q) {
                const int it = wave + q * NW;
                if (it >= n_items) break;
                float acc = 0.0f;
#pragma unroll
                for (int r = 0; r < NVR; ++r) {
                    const uint4 xr = xlds[((it % kParts) * NVR + r) * kWave + lane];
                    acc = dot2(xr.x, rw[q][r].x, acc);
                    acc = dot2(xr.y, rw[q][r].y, acc);
                    acc = dot2(xr.z, rw[q][r].z, acc);
                    acc = dot2(xr.w, rw[q][r].w, acc);
                }
                acc = group_reduce_sum_to_last<64>(acc);
                if (lane == kWave - 1) plog[it] = acc;
            }
            FLOE_TL(1);
            __syncthreads();
            const int l16 = lane & 15;
            if (producer && l16 < ro.n_experts) lg = plog[2 * l16] + plog[2 * l16 + 1];
        }
        ex = ro.n_experts + (slot - ro.top_k);  // a shared expert
        if (producer) {
            if (ro.top_k > 0) {
                if constexpr (ROUTED == 1) pick = route_pick_wave64(lg, lane, ro.n_experts, ro.top_k);
                else pick = route_pick_wave16(lg, lane, ro.n_experts, ro.top_k);
                if (slot < ro.top_k) ex = __builtin_amdgcn_readlane(pick.id, slot);
            }
            if (lane == 0) lds_poke(&expert_of_queue[wave], ex);
            e = tab[ex];
            tau = taus[ex];
        }
    } else {
        e = task_expert_of(map, task);
        tau = task_tau[task];
        __syncthreads();  // queues, flags and xlds are set up
    }
    FLOE_TL(2);

    if (producer) {
        // ================================================================ producer: codes -> v -> queue
        const int G = d >> gshift;
        const int jw = (blk * kFusedProducers + wave) * nq;
        auto channel_of = [&](int p) {
            const int j = jw + p * CPW + sub;
            return j < f ? j : f - 1;  // keep the address in bounds; a clamped lane's result is not used
        };
        // The codes of a pass travel straight into LDS, into the two result slabs of this producer's own consumers
        // (unused until those have seen the producer's flag); only scale and zero take registers.
        using St = StageTraits<BITS>;
        constexpr bool kStaged = staged_codes<BITS>();
        constexpr int kSlot = stage_slot_bytes<BITS>();
        constexpr int kVmPerPass = St::kPieces + 2;  // requests per pass: the pieces, scale, zero
        unsigned char* stage = reinterpret_cast<unsigned char*>(&yred[kFusedCpp * wave][0]);
        static_assert(!kStaged || kDepth * kSlot <= kFusedCpp * d * 4, "the staging ring must fit the two slabs");
        static_assert(!kStaged || kVmPerPass * (kDepth - 1) < 64, "the wait counts outstanding requests in six bits");
        static_assert(!kStaged || St::kPieces == 1, "one piece per pass is read back ahead");
        UnitLoad<BITS, UPC, G32> ld[kDepth];
        // the lane's part of the three addresses of a pass; the channel's part is a scalar at d = 4096
        const unsigned char* lane_codes = reinterpret_cast<const unsigned char*>(e.codes) + (size_t)u * (BITS * 8);
        const h16* lane_scale = e.scale + (G32 ? 2 * u : (u * 64) >> gshift);
        const h16* lane_zero = e.zero + (G32 ? 2 * u : (u * 64) >> gshift);
        auto issue = [&](int slot, int p) {
            const int j = channel_of(p);
            if constexpr (kStaged) {
                const unsigned char* src = lane_codes + (size_t)j * (UPC * BITS * 8);
#pragma unroll
                for (int pc = 0; pc < St::kPieces; ++pc) dma16_to_lds(src + pc * 16, stage + slot * kSlot + pc * 1024);
                ld[slot].issue_meta_at(lane_scale, lane_zero, (size_t)j * G);
            } else {
                ld[slot].issue(e, j, u, G, gshift);
            }
        };
#pragma unroll
        for (int p = 0; p < kDepth; ++p) {
            issue(p, p);
            __builtin_amdgcn_sched_barrier(0);  // the waits below count requests in exactly this order
        }
        FLOE_TL(3);

        // This lane's 64 activations (the unit it owns in every channel), from the copy in LDS: read from memory,
        // the 128-byte stride between lanes made 512 cache-line requests per wave, all workgroups on the same lines.
        uint32_t raw[32];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint4 q = xlds[u * 8 + r];
            raw[4 * r + 0] = q.x; raw[4 * r + 1] = q.y; raw[4 * r + 2] = q.z; raw[4 * r + 3] = q.w;
        }

        float wgt = 1.0f;
        if (ROUTED) {
            if (ro.top_k > 0) {
                const float wl = route_weight_wave16(pick, ro.top_k, ro.renormalize);
                if (slot < ro.top_k) wgt = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wl), slot));
            }
            if (blk == 0 && tid == 0) {  // the task's routing record (statistics)
                ro.task_table[task] = e;
                ro.task_expert[task] = ex;
                ro.task_weight[task] = wgt;
                ro.task_tau[task] = tau;
            }
        } else if (task_scale) {
            wgt = task_scale[task];
        }

        uint32_t xs[32];
        float Xg[2], Xoff[2];
        // every group of UPC lanes holds the whole token, so the wave-wide maximum is the token's
        const float amax = wave_allreduce_max_nonneg(unit_amax(raw));
        const int down = xprep_down<BITS>(amax);
        const float inv_p = ldexpf(1.0f, down);
        unit_prepare<BITS>(raw, down, xs, Xoff, Xg);
        uint32_t magic = 0x3C003C00u;
        asm volatile("" : "+v"(magic));  // keep it in a VGPR: v_and_or_b32 takes one scalar operand only
        FLOE_TL(4);

        int k = 0;  // entries pushed so far (wave-uniform)
        // Staged codes come back from LDS one pass ahead.  A pass's codes have landed once only the requests made
        // after them are outstanding: kVmPerPass per pass, and kDepth - 1 passes are behind pass p at its own turn,
        // kDepth - 2 behind pass p + 1 at that time.  The counts are the same in every round because the last round
        // keeps requesting (see below).  More may be outstanding - a store of v, say - which only makes a wait longer.
        u32x4 cw_next;
        if constexpr (kStaged) {
            wait_vm_all_but<kVmPerPass * (kDepth - 1)>();
            lds_piece_request(stage + lane * 16, cw_next);
        }
#pragma unroll 1
        for (int p0 = 0; p0 < n_pass; p0 += kDepth) {
#pragma unroll
            for (int i = 0; i < kDepth; ++i) {
                const int p = p0 + i;
                if (!kStaged && p >= n_pass) break;  // last, shorter round (wave-uniform); staged: n_pass % kDepth == 0
                const int j = jw + p * CPW + sub;
                if constexpr (kStaged) {
                    lds_piece_arrived(cw_next);
                    ld[i].cw[0] = cw_next.x; ld[i].cw[1] = cw_next.y; ld[i].cw[2] = cw_next.z; ld[i].cw[3] = cw_next.w;
                    if constexpr (kDepth >= 2) {  // (past the last pass this reads a slot that nobody uses)
                        wait_vm_all_but<kVmPerPass * (kDepth - 2)>();
                        lds_piece_request(stage + ((i + 1) % kDepth) * kSlot + lane * 16, cw_next);
                    }
                }
                // scale and zero stay untouched until here (otherwise their unpacking is hoisted out of the loop for
                // the first round, and with it a wait for every load of that round)
                if constexpr (G32) asm volatile("" : "+v"(ld[i].s), "+v"(ld[i].z));
                else asm volatile("" : "+v"(ld[i].sh), "+v"(ld[i].zh));
                float part = unit_value<BITS, UPC, G32>(ld[i], xs, Xoff, Xg, magic);
                if constexpr (kStaged) {
                    // In the last round there is nothing left to request; the slot asks for the final pass again
                    // (a cache hit that nobody reads) so that every round has the same, unconditional sequence of
                    // requests: with a condition here the compiler has to assume that no request follows and makes
                    // each round wait for all of its loads at once.
                    const int pn = p + kDepth < n_pass ? p + kDepth : n_pass - 1;
                    issue(i, pn);
                } else {
                    if (p + kDepth < n_pass) issue(i, p + kDepth);
                }
                part = group_reduce_sum_to_last<UPC>(part) * inv_p;
                const bool mine = u == UPC - 1 && p < n_pass && j < f;
                if (v_out && mine) v_out[(size_t)task * f + j] = part;
                const bool hit = mine && fabsf(part) > tau;
                unsigned long long hits = __ballot(hit);
                while (hits) {  // wave-uniform; ascending channel order
                    const int bit = __ffsll((long long)hits) - 1;
                    hits &= hits - 1;
                    if (lane == bit) {
                        // the same lane writes both words; LDS keeps a wave's accesses in order, so whoever sees
                        // the channel id also sees the value
                        lds_poke(&qh[wave][k], part * wgt);
                        lds_poke(&qj[wave][k], j);
                    }
                    ++k;
                }
                __builtin_amdgcn_sched_barrier(0);  // keep the request for pass p + kDepth where it is
            }
        }
        if constexpr (kStaged) lds_piece_arrived(cw_next);  // the read-ahead of the last pass: its registers are free only now
        if constexpr (kStaged) wait_vm_all_but<0>();  // the ring lies in the consumers' result slabs: nothing may land later
        if (lane == 0) {
            lds_poke(&done[wave], 1);  // after the last push, in program order
            atomicAdd(&n_sel, k);
        }
        FLOE_TL(5);
    } else {
        // ================================================================ consumer: queue -> chunk -> y
        const int c = wave - kFusedProducers;   // consumer id: serves queue c / kFusedCpp, entries c % kFusedCpp, + kFusedCpp, ...
        const int qc = c / kFusedCpp;
        if (ROUTED) {  // the producer of this queue publishes its expert right after the pick
            int exq;
            while ((exq = __builtin_amdgcn_readfirstlane(lds_peek(&expert_of_queue[qc]))) < 0) __builtin_amdgcn_s_sleep(4);
            e = tab[exq];
        }
        float acc[8 * NV];
#pragma unroll
        for (int i = 0; i < 8 * NV; ++i) acc[i] = 0.0f;
        int k = c % kFusedCpp;
        while (k < nq) {  // the queue cannot hold more than its producer has channels
            // The wait is a loop of its own that touches no accumulator: as a second way back to the head of the
            // outer loop it made the compiler copy all of them (64 moves) on every empty poll.
            int j;
            for (;;) {
                j = __builtin_amdgcn_readfirstlane(lds_peek(&qj[qc][k]));
                if (j >= 0) break;
                if (__builtin_amdgcn_readfirstlane(lds_peek(&done[qc])) != 0) {
                    // the flag is raised after the last push: look once more, then the queue is known to be empty
                    j = __builtin_amdgcn_readfirstlane(lds_peek(&qj[qc][k]));
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
            if (j < 0) break;
            const float h0 = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(lds_peek(reinterpret_cast<const int*>(&qh[qc][k]))));
            const uint4* gp = reinterpret_cast<const uint4*>(e.gd + (size_t)j * 2 * d);
            uint4 gv[NV], dv[NV];
#pragma unroll
            // (plain loads on purpose: measured 5 us faster here than loads typed as global memory)
            for (int r = 0; r < NV; ++r) gv[r] = gp[r * kWave + lane];
#pragma unroll
            for (int r = 0; r < NV; ++r) dv[r] = gp[(d / 8) + r * kWave + lane];
            float g = 0.0f;
#pragma unroll
            for (int r = 0; r < NV; ++r) {
                const uint4 xr = xlds[r * kWave + lane];
                g = dot2(xr.x, gv[r].x, g);
                g = dot2(xr.y, gv[r].y, g);
                g = dot2(xr.z, gv[r].z, g);
                g = dot2(xr.w, gv[r].w, g);
            }
            g = wave_allreduce_sum(g);
            const float h = silu(g) * h0;
#pragma unroll
            for (int r = 0; r < NV; ++r) {
                const uint32_t wds[4] = {dv[r].x, dv[r].y, dv[r].z, dv[r].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const h16x2 pr = as_h2(wds[q]);
                    acc[r * 8 + 2 * q + 0] = fmaf(h, (float)pr.x, acc[r * 8 + 2 * q + 0]);
                    acc[r * 8 + 2 * q + 1] = fmaf(h, (float)pr.y, acc[r * 8 + 2 * q + 1]);
                }
            }
            k += kFusedCpp;
        }
        // The producer's staging ring lies in this consumer's result slab.  A consumer that left the loop because its
        // queue was full to capacity (every channel of the block selected) has not seen the producer's flag yet, and
        // direct-to-LDS loads of the producer may still be on their way: the slab is written only after the flag,
        // which the producer raises behind its last wait.
        if constexpr (staged_codes<BITS>()) {
            while (__builtin_amdgcn_readfirstlane(lds_peek(&done[qc])) == 0) __builtin_amdgcn_s_sleep(1);
        }
        // lane owns columns [(r * 64 + lane) * 8, + 8)
#pragma unroll
        for (int r = 0; r < NV; ++r) {
            float4* o4 = reinterpret_cast<float4*>(&yred[c][(r * kWave + lane) * 8]);
            o4[0] = make_float4(acc[r * 8 + 0], acc[r * 8 + 1], acc[r * 8 + 2], acc[r * 8 + 3]);
            o4[1] = make_float4(acc[r * 8 + 4], acc[r * 8 + 5], acc[r * 8 + 6], acc[r * 8 + 7]);
        }
        FLOE_TL_AT(6, kFusedProducers * 64);
    }
    __syncthreads();
    FLOE_TL(7);
    // ---- the workgroup's partial y: consumers summed in a fixed order
    float4* out = reinterpret_cast<float4*>(partial + ((size_t)task * gridDim.x + blk) * d);
    for (int c4 = tid; c4 < d / 4; c4 += kFusedThreads) {
        float4 s = reinterpret_cast<const float4*>(&yred[0][0])[c4];
#pragma unroll
        for (int c = 1; c < kFusedConsumers; ++c) {
            const float4 a = reinterpret_cast<const float4*>(&yred[c][0])[c4];
            s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
        }
        out[c4] = s;
    }
    if (tid == 0) wg_count[(size_t)task * gridDim.x + blk] = n_sel;
    FLOE_TL(8);
}

// ---- launch: bits fixed by the translation unit, the rest chosen here
template <int BITS, int UPC, bool G32>
static hipError_t fused_launch_shape(const FusedArgs& a, int gshift, hipStream_t stream) {
    const dim3 grid(fused_blocks(a.d, a.f, a.passes), a.n_tasks), block(kFusedThreads);
    const RouteArgs ro = a.route ? *a.route : RouteArgs{};
    // passes in flight per producer wave: INT2 stages 14 KB of codes in LDS, as far as the ring fits the two result
    // slabs it borrows (8 d bytes); INT3 and INT4 hold 4 passes in registers (8 / 10 per pass)
    constexpr int kWant = BITS == 2 ? 14 : 7;
    constexpr int kFit = staged_codes<BITS>() ? kFusedCpp * UPC * 64 * 4 / stage_slot_bytes<BITS>() : 4;
    constexpr int kDepth = staged_codes<BITS>() ? (kWant < kFit ? kWant : kFit) : 4;
    // a.passes passes per producer at run time; the template argument only sizes the queues and caps the depth
    if (a.passes < kFusedMinPasses || a.passes > kFusedMaxPasses) return hipErrorInvalidValue;  // (the grid follows a.passes)
    static_assert(kDepth == fused_depth(UPC * 64, BITS), "the host rounds the pass count to this depth");
    constexpr int kDepthSmall = kDepth < kFusedMinPasses ? kDepth : kFusedMinPasses;
    // staged codes: whole rounds of the ring (the waits in the kernel count on it)
    if (staged_codes<BITS>() && a.passes % (a.passes <= kFusedMinPasses ? kDepthSmall : kDepth) != 0) return hipErrorInvalidValue;
#define FLOE_FUSED_GO(ROUTED, P)                                                                                 \
    fused_ffn_kernel<BITS, UPC, G32, ROUTED, P, (kDepth < P ? kDepth : P)><<<grid, block, 0, stream>>>(a.map, a.x, ro, a.task_tau,   \
                                                                                    a.task_scale, a.f, a.passes, gshift, \
                                                                                    a.v_out, a.partial, a.wg_count)
#define FLOE_FUSED_PASSES(ROUTED)                                               \
    if (a.passes <= kFusedMinPasses) {                                          \
        FLOE_FUSED_GO(ROUTED, kFusedMinPasses);                                 \
    } else {                                                                    \
        FLOE_FUSED_GO(ROUTED, kFusedMaxPasses);                                 \
    }
    if (a.route) {
        if (a.route->top_k < 1 || a.route->top_k + a.route->n_shared > 16 ||
            a.route->n_experts > (a.route->logits ? kFusedMaxRouted : 16))
            return hipErrorInvalidValue;
        if (a.route->logits) {
            FLOE_FUSED_PASSES(1)
        } else {
            FLOE_FUSED_PASSES(2)
        }
    } else {
        FLOE_FUSED_PASSES(0)
    }
#undef FLOE_FUSED_PASSES
#undef FLOE_FUSED_GO
    return hipGetLastError();
}

template <int BITS>
static hipError_t fused_launch_bits(const FusedArgs& a, hipStream_t stream) {
    if (a.f == 0 || a.n_tasks == 0) return hipSuccess;
    int gshift = 0;
    while ((1 << gshift) < a.group) ++gshift;
    const bool g32 = a.group == 32;
    switch (a.d) {
        case 4096: return g32 ? fused_launch_shape<BITS, 64, true>(a, gshift, stream) : fused_launch_shape<BITS, 64, false>(a, gshift, stream);
        case 2048: return g32 ? fused_launch_shape<BITS, 32, true>(a, gshift, stream) : fused_launch_shape<BITS, 32, false>(a, gshift, stream);
        case 1024: return g32 ? fused_launch_shape<BITS, 16, true>(a, gshift, stream) : fused_launch_shape<BITS, 16, false>(a, gshift, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace floe
