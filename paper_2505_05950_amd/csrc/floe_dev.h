// Device-side helpers shared by the gfx950 kernels of the FloE decode path (wave64, CDNA4).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace floe {

typedef _Float16 h16;
typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// One compressed expert as the kernels see it (HBM-resident pointer table entry, 32 bytes).
struct DevExpert {
    const uint32_t* codes;
    const h16* scale;
    const h16* zero;
    const h16* gd;
};

// How a kernel finds the data of "task" q = (token, slot): either every task uses `single`
// (one-expert entry points) or the router has written one resolved entry per task into task_table.
struct TaskMap {
    DevExpert single;
    const DevExpert* task_table;  // nullptr => use `single`; else [n_tasks], written by the router kernel
    int32_t slots;                // tasks per token; token of task q is q / slots
};

// Pointers that a kernel reads out of a table (HBM or LDS) carry no address space for the compiler, which then
// emits FLAT loads: those also count against the LDS counter, so every wait for an LDS result would wait for the
// weight loads in flight.  All matrices of an expert live in global memory; these loads say so.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#define FLOE_GLOBAL __attribute__((address_space(1)))
__device__ __forceinline__ uint4 gload16(const void* p) {
    const u32x4 q = *(const FLOE_GLOBAL u32x4*)p;
    return make_uint4(q.x, q.y, q.z, q.w);
}
__device__ __forceinline__ uint2 gload8(const void* p) {
    const u32x2 q = *(const FLOE_GLOBAL u32x2*)p;
    return make_uint2(q.x, q.y);
}
__device__ __forceinline__ uint32_t gload4(const void* p) { return *(const FLOE_GLOBAL uint32_t*)p; }
__device__ __forceinline__ uint32_t gload2(const void* p) { return *(const FLOE_GLOBAL uint16_t*)p; }
__device__ __forceinline__ _Float16 gloadh(const void* p) { return *(const FLOE_GLOBAL _Float16*)p; }
__device__ __forceinline__ float gloadf(const void* p) { return *(const FLOE_GLOBAL float*)p; }

__device__ __forceinline__ DevExpert task_expert_of(const TaskMap& m, int task) {
    if (m.task_table == nullptr) return m.single;
    return m.task_table[task];
}

__device__ __forceinline__ h16x2 as_h2(uint32_t u) { return __builtin_bit_cast(h16x2, u); }
__device__ __forceinline__ uint32_t as_u32(h16x2 h) { return __builtin_bit_cast(uint32_t, h); }

// acc + a.x*b.x + a.y*b.y with an fp32 accumulator (v_dot2c_f32_f16)
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2(as_h2(a), as_h2(b), acc, false);
}

// (a & mask) | magic in one VALU instruction; mask must be wave-uniform (it is read from an SGPR)
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t magic) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(magic));
    return r;
}

// ---- cross-lane sums on the DPP path (no LDS traffic) -------------------------------------------
// DPP control words of gfx9: row_ror:n = 0x120 + n, row_bcast:15 = 0x142, row_bcast:31 = 0x143.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
    const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xF, false);
    return x + __builtin_bit_cast(float, y);
}

// every lane receives the sum over its row of 16 lanes
__device__ __forceinline__ float row16_allreduce_sum(float x) {
    x = dpp_add<0x128, 0xF>(x);
    x = dpp_add<0x124, 0xF>(x);
    x = dpp_add<0x122, 0xF>(x);
    x = dpp_add<0x121, 0xF>(x);
    return x;
}

// Sum over groups of WIDTH consecutive lanes (16, 32 or 64).  The total is valid in the LAST lane of
// each group (lane % WIDTH == WIDTH - 1); other lanes hold partial sums.
template <int WIDTH>
__device__ __forceinline__ float group_reduce_sum_to_last(float x) {
    static_assert(WIDTH == 16 || WIDTH == 32 || WIDTH == 64, "group width");
    x = row16_allreduce_sum(x);
    if (WIDTH >= 32) x = dpp_add<0x142, 0xA>(x);  // rows 1 and 3 += last lane of rows 0 and 2
    if (WIDTH == 64) x = dpp_add<0x143, 0xC>(x);  // rows 2 and 3 += lane 31
    return x;
}

// sum over the 64 lanes, returned to every lane (through a scalar register)
__device__ __forceinline__ float wave_allreduce_sum(float x) {
    x = group_reduce_sum_to_last<64>(x);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

// value of lane (lane rotated right by N inside its row of 16) -- a pure register move, no LDS
template <int CTRL>
__device__ __forceinline__ float dpp_movf(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_movi(int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, false);
}

// max over the row of 16 lanes, delivered to every lane of the row
__device__ __forceinline__ float row16_allreduce_max(float x) {
    x = fmaxf(x, dpp_movf<0x128>(x));
    x = fmaxf(x, dpp_movf<0x124>(x));
    x = fmaxf(x, dpp_movf<0x122>(x));
    x = fmaxf(x, dpp_movf<0x121>(x));
    return x;
}

// max over the 64 lanes (x >= 0 everywhere), returned to every lane
__device__ __forceinline__ float wave_allreduce_max_nonneg(float x) {
    x = row16_allreduce_max(x);
    // lanes that a row_bcast does not write receive 0, which is neutral for non-negative inputs
    x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x142, 0xA, 0xF, false)));
    x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x143, 0xC, 0xF, false)));
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

// Optional phase timeline for tuning builds (-DFLOE_TIMELINE): thread 0 of each workgroup stamps the
// constant 100 MHz clock into g_timeline[wg * 16 + slot].  Compiled out of the product library.
#ifdef FLOE_TIMELINE
static __device__ unsigned long long* g_timeline = nullptr;  // one copy per translation unit
#define FLOE_TL_AT(slot, thread)                                                                           \
    do {                                                                                                   \
        if (g_timeline && threadIdx.x == (thread))                                                         \
            g_timeline[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 16 + (slot)] = wall_clock64();      \
    } while (0)
#else
#define FLOE_TL_AT(slot, thread) \
    do {                         \
    } while (0)
#endif
#define FLOE_TL(slot) FLOE_TL_AT(slot, 0)

__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

}  // namespace floe
