// S7: compact transfer of the selected channels (Sec. 3.4.2).  The paper packs the selected
// [gate column | down row] chunks on the CPU into a pinned buffer and issues asynchronous copies.
// Here the index list lives in HBM, so a copy kernel on a side stream pulls the 4*d-byte chunks straight
// out of pinned, device-mapped host memory with 128-bit loads: no index round trip and no CPU packing.
#include <atomic>

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

// Layer form: the source matrix, list and destination slab are each task's own.  The rows of all tasks form one
// sequence that the waves of the launch walk together: lists of unequal length (the misses of a wrongly and of a
// rightly predicted expert) keep every wave busy to the end, which a link that a few dozen waves saturate needs.
constexpr int kStageTaskBatch = 1024;
__global__ __launch_bounds__(256) void stage_tasks_kernel(const DevExpert* __restrict__ task_table, int vec_per_chunk,
                                                          int f, const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ count, int capacity_rows,
                                                          uint4* __restrict__ dst, int32_t* __restrict__ overflow,
                                                          const int32_t* __restrict__ dst_rows, int n_tasks) {
    __shared__ int first[kStageTaskBatch + 1];  // rows to move of the tasks before this one (within the batch)
    const int tid = threadIdx.x, lane = tid & 63;
    const int gw = blockIdx.x * 4 + (tid >> 6);
    const int nw = gridDim.x * 4;
    for (int t0 = 0; t0 < n_tasks; t0 += kStageTaskBatch) {
        const int nb = min(kStageTaskBatch, n_tasks - t0);
        __syncthreads();  // the previous batch's table is no longer read
        for (int q = tid; q < nb; q += 256) {
            const int n = count[t0 + q];
            first[q + 1] = max(0, min(dst_rows ? n : min(n, capacity_rows), f));  // a list holds at most f entries
            if (!dst_rows && overflow && blockIdx.x == 0) overflow[t0 + q] = n > capacity_rows ? 1 : 0;
        }
        __syncthreads();
        if (tid == 0) {
            first[0] = 0;
            for (int q = 0; q < nb; ++q) first[q + 1] += first[q];
        }
        __syncthreads();
        const int total = first[nb];
        for (int g = gw; g < total; g += nw) {
            int lo = 0, hi = nb - 1;  // the task with first[q] <= g < first[q + 1]
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (first[mid] <= g) lo = mid; else hi = mid - 1;
            }
            const int task = t0 + lo, k = g - first[lo];
            const int j = idx[(size_t)task * f + k];
            if ((unsigned)j >= (unsigned)f) continue;  // never read outside the host matrix
            const int r = dst_rows ? dst_rows[(size_t)task * f + k] : k;
            if (r < 0) continue;
            const uint4* s = reinterpret_cast<const uint4*>(task_table[task].gd) + (size_t)j * vec_per_chunk;
            uint4* o = (dst_rows ? dst : dst + (size_t)task * capacity_rows * vec_per_chunk) + (size_t)r * vec_per_chunk;
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
}

// Workgroups of a copy kernel (all tasks together).  A read of host memory keeps its slot in the memory pipeline for
// microseconds; more of them in flight than the link can use only stand in the way of the HBM reads of kernels that
// run beside the copy.
static std::atomic<int> g_stage_wgs{0};
int stage_workgroups() {
    const int n = g_stage_wgs.load(std::memory_order_relaxed);
    return n > 0 ? n : kStageWorkgroupsDefault;
}
void set_stage_workgroups(int n) { g_stage_wgs.store(n, std::memory_order_relaxed); }

hipError_t launch_stage_tasks(const DevExpert* task_table, int d, int f, const int32_t* idx, const int32_t* count,
                              int capacity_rows, h16* dst, int32_t* overflow, int n_tasks, hipStream_t stream,
                              const int32_t* dst_rows) {
    if (n_tasks == 0) return hipSuccess;
    stage_tasks_kernel<<<dim3(stage_workgroups()), dim3(256), 0, stream>>>(task_table, d / 4, f, idx, count, capacity_rows,
                                                                          reinterpret_cast<uint4*>(dst), overflow, dst_rows,
                                                                          n_tasks);
    return hipGetLastError();
}

hipError_t launch_stage(const h16* host_gd_dev, int d, int f, const int32_t* idx, const int32_t* count, int capacity_rows,
                        h16* dst, int32_t* overflow, hipStream_t stream) {
    const int vec_per_chunk = d / 4;  // 2 * d halves = 4 * d bytes = d / 4 uint4
    stage_kernel<<<dim3(stage_workgroups()), dim3(256), 0, stream>>>(reinterpret_cast<const uint4*>(host_gd_dev), vec_per_chunk, f,
                                                         idx, count, capacity_rows, reinterpret_cast<uint4*>(dst),
                                                         overflow);
    return hipGetLastError();
}

}  // namespace floe
