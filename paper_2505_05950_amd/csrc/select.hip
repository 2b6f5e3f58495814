// S3: mask = |v| > tau, ascending index list and its length (Alg. 1 line 3; S_t of Eq. 5 with the strict
// comparison Alg. 1 uses).  One workgroup of 16 waves per task.  Each wave owns a contiguous slice of
// the channels: pass 1 counts with wave ballots, an LDS prefix over the 16 wave totals gives every wave
// its base offset, pass 2 repeats the ballots and writes each selected channel at
// base + (selected channels before it), which keeps the list ascending without any sort.
#include "floe_dev.h"
#include "launch.h"

namespace floe {

__global__ __launch_bounds__(1024) void select_kernel(const float* __restrict__ v, int f, const float* __restrict__ tau,
                                                      int32_t* __restrict__ idx, int32_t* __restrict__ count) {
    constexpr int kWaves = 16;
    __shared__ int wave_total[kWaves];
    const int task = blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const float th = tau[task];
    const float* vt = v + (size_t)task * f;
    int32_t* it = idx + (size_t)task * f;
    // slice of this wave: a multiple of 64 channels
    const int chunks = (f + kWave - 1) / kWave;
    const int chunks_per_wave = (chunks + kWaves - 1) / kWaves;
    const int c0 = wave * chunks_per_wave;
    const int c1 = min(chunks, c0 + chunks_per_wave);

    int total = 0;
    for (int c = c0; c < c1; ++c) {
        const int j = c * kWave + lane;
        const bool keep = j < f && fabsf(vt[j]) > th;
        total += __popcll(__ballot(keep));
    }
    if (lane == 0) wave_total[wave] = total;
    __syncthreads();
    int base = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int n = wave_total[w];
        base += w < wave ? n : 0;
        all += n;
    }
    if (tid == 0) count[task] = all;
    const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    for (int c = c0; c < c1; ++c) {
        const int j = c * kWave + lane;
        const bool keep = j < f && fabsf(vt[j]) > th;
        const uint64_t m = __ballot(keep);
        if (keep) it[base + __popcll(m & below)] = j;
        base += __popcll(m);
    }
}

hipError_t launch_select(const float* v, int f, int n_tasks, const float* tau, int32_t* idx, int32_t* count,
                         hipStream_t stream) {
    if (n_tasks == 0) return hipSuccess;
    select_kernel<<<dim3(n_tasks), dim3(1024), 0, stream>>>(v, f, tau, idx, count);
    return hipGetLastError();
}

}  // namespace floe
