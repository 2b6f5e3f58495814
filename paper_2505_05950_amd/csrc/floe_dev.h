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
// (one-expert entry points) or the expert id is looked up in task_expert and resolved in `table`.
struct TaskMap {
    DevExpert single;
    const DevExpert* table;     // nullptr => use `single`
    const int32_t* task_expert; // [n_tasks] expert id per task (layer path)
    int32_t slots;              // tasks per token; token of task q is q / slots
};

__device__ __forceinline__ DevExpert task_expert_of(const TaskMap& m, int task) {
    if (m.table == nullptr) return m.single;
    return m.table[m.task_expert[task]];
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

// Sum over the `width` consecutive lanes that share lane / width (width a power of two <= 64);
// every lane of the group receives the total.
template <int WIDTH>
__device__ __forceinline__ float group_allreduce_sum(float x) {
#pragma unroll
    for (int o = WIDTH / 2; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
    return x;
}

__device__ __forceinline__ float wave_allreduce_sum(float x) { return group_allreduce_sum<kWave>(x); }

__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

}  // namespace floe
