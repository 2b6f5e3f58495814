// Bookkeeping for prefetching the next layer's channels (intra-expert reuse of Sec. 3.3: the hidden state in
// front of layer i stands in for the one in front of layer i + 1, the up projection of layer i + 1 applied to it
// predicts which channels will pass the threshold, and their [gate | down] chunks are copied ahead of time).
// When the layer's real input arrives, only the channels that were not predicted still have to cross the bus.
//
//   rowmap_kernel      after the predicted chunks have been staged: row_of[q][j] = staging row of channel j
//   match_rows_kernel  with the real lists: where does each selected channel sit, which ones are missing
#include "floe_dev.h"
#include "launch.h"

namespace floe {

// one workgroup per predicted task
__global__ __launch_bounds__(1024) void rowmap_kernel(const int32_t* __restrict__ idx, const int32_t* __restrict__ count,
                                                      const int32_t* __restrict__ task_expert, int f,
                                                      int capacity_rows, int32_t* __restrict__ row_of,
                                                      int32_t* __restrict__ pred_expert,
                                                      int32_t* __restrict__ pred_count) {
    const int q = blockIdx.x;
    int32_t* map = row_of + (size_t)q * f;
    const int32_t* list = idx + (size_t)q * f;
    const int K = min(min(count[q], capacity_rows), f);
    for (int j = threadIdx.x; j < f; j += blockDim.x) map[j] = -1;
    __syncthreads();  // the fill is complete before the scatter (same workgroup; the barrier orders global memory too)
    for (int k = threadIdx.x; k < K; k += blockDim.x) {
        const int j = list[k];
        if ((unsigned)j < (unsigned)f) map[j] = k;
    }
    if (threadIdx.x == 0) {
        pred_expert[q] = task_expert[q];
        pred_count[q] = K;
    }
}

// one workgroup (256 threads) per actual task
__global__ __launch_bounds__(256) void match_rows_kernel(const int32_t* __restrict__ idx, const int32_t* __restrict__ count,
                                                         const int32_t* __restrict__ task_expert, int f, int slots,
                                                         int capacity_rows, int n_tasks,
                                                         const int32_t* __restrict__ row_of,
                                                         const int32_t* __restrict__ pred_expert,
                                                         const int32_t* __restrict__ pred_count,
                                                         int32_t* __restrict__ rows, int32_t* __restrict__ miss_idx,
                                                         int32_t* __restrict__ miss_rows,
                                                         int32_t* __restrict__ miss_count,
                                                         int32_t* __restrict__ overflow, PrefetchStat* __restrict__ stat,
                                                         const int32_t* __restrict__ expert_row_of, int miss_first_row) {
    __shared__ int wave_tot[4];
    __shared__ int hit_tot[4];
    const int q = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int t = q / slots;
    const int ex = task_expert[q];
    // Resident-channel cache (expert_row_of given): the map is the expert's own, its entries are rows of the whole pool,
    // and the task's fresh rows are its slab behind the resident part of the pool.
    const bool cache = expert_row_of != nullptr;
    // Prefetch: the predicted task of the same token that loaded this expert, if any (slots <= 64: every thread scans)
    int qp = -1;
    if (!cache)
        for (int s = 0; s < slots; ++s)
            if (qp < 0 && pred_expert[t * slots + s] == ex) qp = t * slots + s;
    const bool matched = cache || qp >= 0;
    const int slab = cache ? q : (matched ? qp : n_tasks + q);   // spare slabs follow the predicted ones
    const int base = (!cache && matched) ? pred_count[qp] : 0;   // fresh rows go behind the predicted ones
    const int32_t* map = cache ? expert_row_of + (size_t)ex * f : (matched ? row_of + (size_t)qp * f : nullptr);
    const int slab_row0 = cache ? miss_first_row + slab * capacity_rows : slab * capacity_rows;
    const int32_t* list = idx + (size_t)q * f;
    int32_t* out_rows = rows + (size_t)q * f;
    int32_t* out_mi = miss_idx + (size_t)q * f;
    int32_t* out_mr = miss_rows + (size_t)q * f;
    const int K = min(count[q], f);
    int n_miss = 0, n_hit = 0, dropped = 0;
    for (int k0 = 0; k0 < K; k0 += 256) {
        const int k = k0 + tid;
        int j = -1, r = -1;
        if (k < K) {
            j = list[k];
            if ((unsigned)j >= (unsigned)f) j = -1;
            if (j >= 0 && map) r = map[j];
        }
        const bool hit = j >= 0 && r >= 0;
        const bool miss = j >= 0 && r < 0;
        // ascending rank of this thread's miss inside the chunk of 256
        const unsigned long long mb = __ballot(miss), hb = __ballot(hit);
        const int before = __popcll(mb & ((1ull << lane) - 1ull));
        if (lane == 0) {
            wave_tot[wave] = __popcll(mb);
            hit_tot[wave] = __popcll(hb);
        }
        __syncthreads();
        int off = 0, tot = 0, hits = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            off += w < wave ? wave_tot[w] : 0;
            tot += wave_tot[w];
            hits += hit_tot[w];
        }
        if (k < K) {
            int row = -1;
            if (hit) {
                row = cache ? r : slab_row0 + r;
            } else if (miss) {
                const int m = n_miss + off + before;
                const int fresh = base + m;
                if (fresh < capacity_rows) row = slab_row0 + fresh;
                out_mi[m] = j;          // listed even when it does not fit: its row is -1 and nothing is copied
                out_mr[m] = row;
            }
            out_rows[k] = row;
        }
        n_miss += tot;
        n_hit += hits;
        __syncthreads();  // wave_tot is rewritten by the next chunk
    }
    if (tid == 0) {
        dropped = base + n_miss > capacity_rows ? 1 : 0;
        miss_count[q] = n_miss;
        if (overflow) overflow[q] = dropped;
        if (stat) {
            PrefetchStat s;
            s.expert_predicted = matched ? 1 : 0;
            s.predicted = (!cache && matched) ? pred_count[qp] : 0;
            s.hits = n_hit;
            s.misses = n_miss;
            stat[q] = s;
        }
    }
}

hipError_t launch_rowmap(const int32_t* idx, const int32_t* count, const int32_t* task_expert, int f, int capacity_rows,
                         int32_t* row_of, int32_t* pred_expert, int32_t* pred_count, int n_tasks, hipStream_t stream) {
    if (n_tasks == 0) return hipSuccess;
    rowmap_kernel<<<dim3(n_tasks), dim3(1024), 0, stream>>>(idx, count, task_expert, f, capacity_rows, row_of, pred_expert,
                                                           pred_count);
    return hipGetLastError();
}

hipError_t launch_match_rows(const int32_t* idx, const int32_t* count, const int32_t* task_expert, int f, int slots,
                             int capacity_rows, const int32_t* row_of, const int32_t* pred_expert,
                             const int32_t* pred_count, int32_t* rows, int32_t* miss_idx, int32_t* miss_rows,
                             int32_t* miss_count, int32_t* overflow, PrefetchStat* stat, int n_tasks,
                             hipStream_t stream, const int32_t* expert_row_of, int miss_first_row) {
    if (n_tasks == 0) return hipSuccess;
    match_rows_kernel<<<dim3(n_tasks), dim3(256), 0, stream>>>(idx, count, task_expert, f, slots, capacity_rows, n_tasks,
                                                              row_of, pred_expert, pred_count, rows, miss_idx, miss_rows,
                                                              miss_count, overflow, stat, expert_row_of, miss_first_row);
    return hipGetLastError();
}

// Resident-channel cache (more memory = more of the experts kept in HBM, Sec. 4.1): the listed channels of one expert
// are copied from its host matrix into rows first_row, first_row + 1, ... of the pool and entered in the expert's map.
__global__ __launch_bounds__(256) void cache_load_kernel(const DevExpert* __restrict__ table, int expert, int vec_per_chunk,
                                                         int f, const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ count, int first_row, int max_rows,
                                                         uint4* __restrict__ pool, int32_t* __restrict__ row_of) {
    const uint4* src = reinterpret_cast<const uint4*>(table[expert].gd);
    const int K = min(min(count[0], max_rows), f);
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
    for (int k = gw; k < K; k += nw) {
        const int j = idx[k];
        if ((unsigned)j >= (unsigned)f) continue;
        const uint4* s = src + (size_t)j * vec_per_chunk;
        uint4* o = pool + (size_t)(first_row + k) * vec_per_chunk;
        for (int i = lane; i < vec_per_chunk; i += kWave) o[i] = s[i];
        if (lane == 0) row_of[(size_t)expert * f + j] = first_row + k;
    }
}

hipError_t launch_cache_load(const DevExpert* table, int expert, int d, int f, const int32_t* idx, const int32_t* count,
                             int first_row, int max_rows, h16* pool, int32_t* row_of, hipStream_t stream) {
    cache_load_kernel<<<dim3(num_cus()), dim3(256), 0, stream>>>(table, expert, d / 4, f, idx, count, first_row, max_rows,
                                                                reinterpret_cast<uint4*>(pool), row_of);
    return hipGetLastError();
}

}  // namespace floe
