// S7: compact transfer of the selected channels (Sec. 3.4.2).  The paper packs the selected
// [gate column | down row] chunks on the CPU into a pinned buffer and issues asynchronous copies.
// Here the index list lives in HBM, so a copy kernel on a side stream pulls the 4*d-byte chunks straight
// out of pinned, device-mapped host memory with 128-bit loads: no index round trip and no CPU packing.
#include "floe_dev.h"
#include "launch.h"

namespace floe {

// One wave moves whole chunks; a chunk is 4*d bytes = d/4 uint4, read and written fully coalesced.
__global__ __launch_bounds__(256) void stage_kernel(const uint4* __restrict__ src, int vec_per_chunk, int f,
                                                    const int32_t* __restrict__ idx,
                                                    const int32_t* __restrict__ count, int capacity_rows,
                                                    uint4* __restrict__ dst, int32_t* __restrict__ overflow) {
    const int n = count[0];
    const int K = min(n, capacity_rows);
    if (overflow && blockIdx.x == 0 && threadIdx.x == 0) *overflow = n > capacity_rows ? 1 : 0;
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int nw = gridDim.x * 4;
    for (int k = gw; k < K; k += nw) {
        const int j = idx[k];
        if ((unsigned)j >= (unsigned)f) continue;  // never read outside the host matrix
        const uint4* s = src + (size_t)j * vec_per_chunk;
        uint4* o = dst + (size_t)k * vec_per_chunk;
        for (int i = lane; i < vec_per_chunk; i += 4 * kWave) {
            // four independent loads in flight per lane
            uint4 a = s[i];
            uint4 b = i + kWave < vec_per_chunk ? s[i + kWave] : a;
            uint4 c = i + 2 * kWave < vec_per_chunk ? s[i + 2 * kWave] : a;
            uint4 e = i + 3 * kWave < vec_per_chunk ? s[i + 3 * kWave] : a;
            o[i] = a;
            if (i + kWave < vec_per_chunk) o[i + kWave] = b;
            if (i + 2 * kWave < vec_per_chunk) o[i + 2 * kWave] = c;
            if (i + 3 * kWave < vec_per_chunk) o[i + 3 * kWave] = e;
        }
    }
}

// Layer form: blockIdx.y = task; the source matrix, list and destination slab are the task's own.
__global__ __launch_bounds__(256) void stage_tasks_kernel(const DevExpert* __restrict__ task_table, int vec_per_chunk,
                                                          int f, const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ count, int capacity_rows,
                                                          uint4* __restrict__ dst, int32_t* __restrict__ overflow,
                                                          const int32_t* __restrict__ dst_rows) {
    const int task = blockIdx.y;
    const uint4* src = reinterpret_cast<const uint4*>(task_table[task].gd);
    const int32_t* it = idx + (size_t)task * f;
    uint4* out = dst + (size_t)task * capacity_rows * vec_per_chunk;
    const int32_t* rw = dst_rows ? dst_rows + (size_t)task * f : nullptr;
    const int n = count[task];
    const int K = rw ? min(n, f) : min(n, capacity_rows);
    if (!rw && overflow && blockIdx.x == 0 && threadIdx.x == 0) overflow[task] = n > capacity_rows ? 1 : 0;
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int nw = gridDim.x * 4;
    for (int k = gw; k < K; k += nw) {
        const int j = it[k];
        if ((unsigned)j >= (unsigned)f) continue;
        const int r = rw ? rw[k] : k;
        if (r < 0) continue;
        const uint4* s = src + (size_t)j * vec_per_chunk;
        uint4* o = (rw ? dst : out) + (size_t)r * vec_per_chunk;
        for (int i = lane; i < vec_per_chunk; i += 4 * kWave) {
            uint4 a = s[i];
            uint4 b = i + kWave < vec_per_chunk ? s[i + kWave] : a;
            uint4 c = i + 2 * kWave < vec_per_chunk ? s[i + 2 * kWave] : a;
            uint4 e = i + 3 * kWave < vec_per_chunk ? s[i + 3 * kWave] : a;
            o[i] = a;
            if (i + kWave < vec_per_chunk) o[i + kWave] = b;
            if (i + 2 * kWave < vec_per_chunk) o[i + 2 * kWave] = c;
            if (i + 3 * kWave < vec_per_chunk) o[i + 3 * kWave] = e;
        }
    }
}

hipError_t launch_stage_tasks(const DevExpert* task_table, int d, int f, const int32_t* idx, const int32_t* count,
                              int capacity_rows, h16* dst, int32_t* overflow, int n_tasks, hipStream_t stream,
                              const int32_t* dst_rows) {
    if (n_tasks == 0) return hipSuccess;
    const int nblk = num_cus() / n_tasks > 0 ? num_cus() / n_tasks : 1;
    stage_tasks_kernel<<<dim3(nblk, n_tasks), dim3(256), 0, stream>>>(task_table, d / 4, f, idx, count, capacity_rows,
                                                                     reinterpret_cast<uint4*>(dst), overflow, dst_rows);
    return hipGetLastError();
}

hipError_t launch_stage(const h16* host_gd_dev, int d, int f, const int32_t* idx, const int32_t* count, int capacity_rows,
                        h16* dst, int32_t* overflow, hipStream_t stream) {
    const int vec_per_chunk = d / 4;  // 2 * d halves = 4 * d bytes = d / 4 uint4
    stage_kernel<<<dim3(num_cus()), dim3(256), 0, stream>>>(reinterpret_cast<const uint4*>(host_gd_dev), vec_per_chunk, f,
                                                         idx, count, capacity_rows, reinterpret_cast<uint4*>(dst),
                                                         overflow);
    return hipGetLastError();
}

}  // namespace floe
