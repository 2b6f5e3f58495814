// S4 + S5 for decode batches (Alg. 1 steps 4-5; the paper itself is batch-1, each token keeps its own threshold, mask
// and result): the tokens that were routed to the same expert share ONE read of every [gate | down] chunk
// (Sec. 3.4.2) that any of them selected.  A row of the union serves exactly the tokens whose mask holds it; for the
// others its contribution is an exact zero.
//
// Per expert group (up to 16 tokens of one expert, see group_tokens_kernel) the selected rows form a dense
// (tokens x d) x (d x rows) contraction for the gate and a (tokens x rows) x (rows x d) one for the down projection,
// so both go to the matrix cores; the kernels stay bound by the HBM stream of the rows.
//
//   gate_union_kernel   workgroup = (group, block of channels).  Builds the ascending list of the block's union rows
//                       from the tasks' mask bits (ballot-free: one lane per mask word, prefix sum over the wave),
//                       keeps the group's activations in LDS, and computes A[row][token] = gate_row . x_token with
//                       v_mfma_f32_16x16x32_f16, a wave per tile of 16 rows, the rows streamed from HBM straight
//                       into the A fragments.  h = SiLU(A) * v * weight where the token's mask bit is set, else 0,
//                       is left in memory as two fp16 numbers (h = hi + lo, so that nothing of fp32 is lost) in
//                       exactly the lane order in which the down kernel's matrix instruction wants it.
//   down_union_kernel   workgroup = (group, block, 1024 output columns).  Y[token][col] += h[token][row] * down[row][col]
//                       with v_mfma_f32_16x16x16_f16: a lane fetches 16-byte pieces of four rows, a 4 x 8 transpose in
//                       registers (v_perm_b32) turns them into B fragments, the accumulators never leave the registers,
//                       and the workgroup stores one fp32 partial per live token; S6 (combine_kernel) adds the partials.
#include <atomic>
#include <cmath>

#include "floe_dev.h"
#include "launch.h"

namespace floe {

typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kGateWaves = 8;
constexpr int kDownWaves = 4;
constexpr int kDownColsPerWave = 256;                              // two chunks of 128 columns
constexpr int kDownColsPerWg = kDownWaves * kDownColsPerWave;      // 1024

// channel range of gate block b: whole mask words, the same split in both kernels
__device__ __forceinline__ void union_block_words(int nwords, int nblk, int b, int& w0, int& w1) {
    const int per = (nwords + nblk - 1) / nblk;
    w0 = min(nwords, b * per);
    w1 = min(nwords, w0 + per);
}

// The ascending list of a block's union rows with the token bits of every row -> LDS (wave 0: a lane per mask word, 64
// words per round) and memory (for a separate down kernel); per-task selected counts of the block (statistics).
// s_task / s_w must have been filled (tasks of dead token rows: -1).  Ends with a barrier; returns the number of rows.
__device__ __forceinline__ int union_list(const UnionArgs& a, const TokenGroup* grp, int n_tok, int blk, int* lrow,
                                          uint32_t* lbits, const int* s_task, int* s_count) {
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nwords = mask_words_per_task(a.f);
    int w0, w1;
    union_block_words(nwords, a.nblk_gate, blk, w0, w1);
    if (wave == 0) {
        int base = 0;
        int csum[16];  // per task: selected channels of this block (statistics)
#pragma unroll
        for (int n = 0; n < 16; ++n) csum[n] = 0;
        for (int wb = w0; wb < w1; wb += 64) {
            const int w = wb + lane;
            uint32_t m[16];
            uint32_t u = 0;
            const int wc = w < w1 ? w : w1 - 1;  // every lane loads a valid word; dead lanes and dead tokens are zeroed
#pragma unroll
            for (int n = 0; n < 16; ++n) m[n] = gload4(a.mask_words + (size_t)s_task[n < n_tok ? n : 0] * nwords + wc);
#pragma unroll
            for (int n = 0; n < 16; ++n) {
                m[n] = (n < n_tok && w < w1) ? m[n] : 0u;
                u |= m[n];
            }
#pragma unroll
            for (int n = 0; n < 16; ++n) csum[n] += __popc(m[n]);
            int inc = __popc(u);
            const int mine = inc;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int up = __shfl_up(inc, o, kWave);
                if (lane >= o) inc += up;
            }
            int k = base + inc - mine;
            while (u) {
                const int b = __ffs(u) - 1;
                u &= u - 1;
                uint32_t bits = 0;
#pragma unroll
                for (int n = 0; n < 16; ++n) bits |= ((m[n] >> b) & 1u) << n;
                lrow[k] = w * 32 + b;
                lbits[k] = bits;
                ++k;
            }
            base += __shfl(inc, kWave - 1, kWave);
        }
        if (lane == 0) *s_count = base;
        if (a.count) {  // every (task, block) entry is written, also by a block without channels
#pragma unroll
            for (int n = 0; n < 16; ++n) {
                if (n < n_tok) {  // wave-uniform
                    int c = csum[n];
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, kWave);
                    if (lane == 0) a.count[(size_t)s_task[n] * a.nblk_gate + blk] = c;
                }
            }
        }
    }
    __syncthreads();
    return *s_count;
}

// tasks and combine weights of the group's token rows -> LDS (followed by a barrier)
__device__ __forceinline__ void union_tasks(const UnionArgs& a, const TokenGroup* grp, int n_tok, int* s_task, float* s_w) {
    const int tid = threadIdx.x;
    if (tid < 16) {
        const int task = tid < n_tok ? grp->task[tid] : -1;
        s_task[tid] = task;
        s_w[tid] = task >= 0 ? (a.task_scale ? a.task_scale[task] : 1.0f) : 0.0f;
    }
    __syncthreads();
}

// What the two-kernel variants do first: the group's activations -> LDS (rows of dead tokens repeat token 0: finite
// numbers whose results are dropped), then the block's list, which also goes to memory for the down kernel.
template <int d, int kXStride>
__device__ __forceinline__ int union_prologue(const UnionArgs& a, const TokenGroup* grp, int n_tok, int blk, unsigned char* xl,
                                              int* lrow, uint32_t* lbits, int* s_task, float* s_w, int* s_count) {
    const int tid = threadIdx.x;
    union_tasks(a, grp, n_tok, s_task, s_w);
    static_assert((d / 8) % 64 == 0, "a row is a whole number of wave-wide pieces");
    for (int i0 = tid; i0 < a.nt * (d / 8); i0 += 4 * kGateWaves * 64) {  // four independent pieces in flight per thread
        uint4 q[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = i0 + j * kGateWaves * 64;
            const int n = i / (d / 8), c = i % (d / 8);
            q[j] = make_uint4(0u, 0u, 0u, 0u);
            if (n < a.nt) q[j] = reinterpret_cast<const uint4*>(a.x + (size_t)(s_task[n < n_tok ? n : 0] / a.slots) * d)[c];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = i0 + j * kGateWaves * 64;
            const int n = i / (d / 8), c = i % (d / 8);
            if (n < a.nt) *reinterpret_cast<uint4*>(xl + (size_t)n * kXStride + c * 16) = q[j];
        }
    }
    const int count = union_list(a, grp, n_tok, blk, lrow, lbits, s_task, s_count);
    const size_t gb = (size_t)blockIdx.y * a.nblk_gate + blk;  // (group, block)
    if (tid == 0) a.ucount[gb] = count;
    for (int k = tid; k < count; k += kGateWaves * 64) a.urow[gb * a.cap + k] = lrow[k];
    return count;
}

// ---------------------------------------------------------------------------------------------------------------
// gate
// ---------------------------------------------------------------------------------------------------------------
// NT: token rows kept in LDS (8 or 16, the group chunk).  x rows are padded by 16 bytes so that the sixteen lanes of a
// fragment read (same k, sixteen tokens) fall into different banks.
template <int NV>  // d = 512 * NV
__global__ __launch_bounds__(kGateWaves * 64) void gate_union_kernel(UnionArgs a) {
    constexpr int d = 512 * NV;
    constexpr int kSteps = d / 32;
    constexpr int kXStride = d * 2 + 16;  // bytes
    constexpr int kDepth = 16;            // k-steps of a tile's rows in flight per lane (16 bytes each; 32 measured slower)
    static_assert(kSteps % kDepth == 0, "d is a multiple of 512");
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char* xl = lds;                                                  // [NT][kXStride]
    int* lrow = reinterpret_cast<int*>(lds + (size_t)a.nt * kXStride);        // [cap]
    uint32_t* lbits = reinterpret_cast<uint32_t*>(lrow + a.cap);              // [cap] token bits of the row
    __shared__ int s_task[16];
    __shared__ float s_w[16];
    __shared__ int s_count;

    if ((int)blockIdx.y >= a.n_groups[0]) return;  // the grid is sized for the worst case
    const TokenGroup* grp = a.groups + blockIdx.y;
    const int n_tok = grp->n;
    const DevExpert e = a.table[grp->expert];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int l16 = lane & 15, g = lane >> 4;
    const int blk = blockIdx.x;
    const int count = union_prologue<d, kXStride>(a, grp, n_tok, blk, xl, lrow, lbits, s_task, s_w, &s_count);
    const size_t gb = (size_t)blockIdx.y * a.nblk_gate + blk;  // (group, block)
    const int ntiles = (count + 15) >> 4;

    // ---- a wave per tile of 16 rows; the first k-steps of the wave's next tile are requested during the last steps
    // of the current one (past the wave's last tile the request repeats that tile: a cache hit that nobody reads)
    auto row_ptr = [&](int t) {
        const int kr = min(16 * t + l16, count - 1);  // rows past the end repeat the last one; their bits are 0
        return reinterpret_cast<const unsigned char*>(e.gd) + (size_t)lrow[kr] * (4 * d) + 16 * g;
    };
    uint4 ga[kDepth];
    if (wave < ntiles) {
        const unsigned char* gp0 = row_ptr(wave);
#pragma unroll
        for (int s = 0; s < kDepth; ++s) ga[s] = gload16(gp0 + 64 * s);
    }
    for (int t = wave; t < ntiles; t += kGateWaves) {
        const unsigned char* gp = row_ptr(t);
        const unsigned char* gp_next = row_ptr(t + kGateWaves < ntiles ? t + kGateWaves : t);
        // v and the mask bits of this lane's four (row, token) results
        float vv[4];
        uint32_t bit[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = 16 * t + 4 * g + i;
            const bool live = k < count && l16 < n_tok;
            const int r = lrow[min(k, count - 1)];
            bit[i] = live ? (lbits[min(k, count - 1)] >> l16) & 1u : 0u;
            vv[i] = bit[i] ? gloadf(a.v + (size_t)s_task[l16] * a.f + r) : 0.0f;
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        const unsigned char* xp = xl + (size_t)(l16 < a.nt ? l16 : 0) * kXStride + 16 * g;
#pragma unroll 1
        for (int s0 = 0; s0 < kSteps - kDepth; s0 += kDepth) {
#pragma unroll
            for (int s = 0; s < kDepth; ++s) {
                const uint4 xq = *reinterpret_cast<const uint4*>(xp + 64 * (s0 + s));
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h16x8, ga[s]), __builtin_bit_cast(h16x8, xq),
                                                             acc, 0, 0, 0);
                ga[s] = gload16(gp + 64 * (s0 + kDepth + s));
            }
        }
#pragma unroll
        for (int s = 0; s < kDepth; ++s) {  // last round: the next tile's first steps take the freed registers
            const uint4 xq = *reinterpret_cast<const uint4*>(xp + 64 * (kSteps - kDepth + s));
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h16x8, ga[s]), __builtin_bit_cast(h16x8, xq), acc,
                                                         0, 0, 0);
            ga[s] = gload16(gp_next + 64 * s);
        }
        // lane (l16, g) holds A[row 16t + 4g + i][token l16]
        const float w = s_w[l16];
        uint32_t hi[2], lo[2];
        h16 hh[4], hl[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float h = bit[i] ? silu(acc[i]) * vv[i] * w : 0.0f;
            hh[i] = (h16)h;
            hl[i] = (h16)(h - (float)hh[i]);
        }
        hi[0] = as_u32(h16x2{hh[0], hh[1]}); hi[1] = as_u32(h16x2{hh[2], hh[3]});
        lo[0] = as_u32(h16x2{hl[0], hl[1]}); lo[1] = as_u32(h16x2{hl[2], hl[3]});
        a.hbuf[(gb * (a.cap / 16) + t) * 64 + lane] = make_uint4(hi[0], hi[1], lo[0], lo[1]);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// down
// ---------------------------------------------------------------------------------------------------------------
// one tile of 16 rows as this lane sees it: its h fragment and 16-byte pieces of rows 4g .. 4g+3, two column chunks
struct DownTile {
    uint4 h;
    uint4 q[2][4];
};

__global__ __launch_bounds__(kDownWaves * 64) void down_union_kernel(UnionArgs a, int d) {
    if ((int)blockIdx.y >= a.n_groups[0]) return;
    const TokenGroup* grp = a.groups + blockIdx.y;
    const int n_tok = grp->n;
    const DevExpert e = a.table[grp->expert];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int l16 = lane & 15, g = lane >> 4;
    const int col0 = blockIdx.z * kDownColsPerWg + wave * kDownColsPerWave;  // this wave's first output column
    const bool wave_live = col0 < d;                                         // (d is a multiple of 512)
    const int ncw = wave_live ? min(2, (d - col0) / 128) : 0;                // chunks of 128 columns in this wave

    f32x4 acc[2][8];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[c][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int per = a.nblk_gate / a.nblk_down;  // gate blocks per down block
    extern __shared__ __align__(16) int lrow[];  // [cap] rows of the current gate block
    for (int gbk = blockIdx.x * per; gbk < (int)(blockIdx.x + 1) * per; ++gbk) {
        const size_t gb = (size_t)blockIdx.y * a.nblk_gate + gbk;
        const int count = a.ucount[gb];
        const int ntiles = (count + 15) >> 4;
        __syncthreads();  // the previous block's list is no longer read
        for (int k = tid; k < count; k += kDownWaves * 64) lrow[k] = a.urow[gb * a.cap + k];
        __syncthreads();
        if (wave_live && ntiles > 0) {
            const uint4* hb = a.hbuf + gb * (a.cap / 16) * 64;
            // every request is unconditional: past the last tile it repeats that tile (cache hits that nobody reads)
            auto load_tile = [&](DownTile& tl, int t) {
                t = t < ntiles ? t : ntiles - 1;
                tl.h = hb[(size_t)t * 64 + lane];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = lrow[min(16 * t + 4 * g + i, count - 1)];
                    const unsigned char* dp = reinterpret_cast<const unsigned char*>(e.gd) + (size_t)row * (4 * d) + 2 * d +
                                              2 * (col0 + 8 * l16);
#pragma unroll
                    for (int c = 0; c < 2; ++c) tl.q[c][i] = gload16(dp + 256 * (c < ncw ? c : 0));
                }
            };
            auto compute_tile = [&](const DownTile& tl) {
                const h16x4 hhi = __builtin_bit_cast(h16x4, make_uint2(tl.h.x, tl.h.y));
                const h16x4 hlo = __builtin_bit_cast(h16x4, make_uint2(tl.h.z, tl.h.w));
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    if (c >= ncw) break;  // wave-uniform
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const uint32_t r0 = p == 0 ? tl.q[c][0].x : (p == 1 ? tl.q[c][0].y : (p == 2 ? tl.q[c][0].z : tl.q[c][0].w));
                        const uint32_t r1 = p == 0 ? tl.q[c][1].x : (p == 1 ? tl.q[c][1].y : (p == 2 ? tl.q[c][1].z : tl.q[c][1].w));
                        const uint32_t r2 = p == 0 ? tl.q[c][2].x : (p == 1 ? tl.q[c][2].y : (p == 2 ? tl.q[c][2].z : tl.q[c][2].w));
                        const uint32_t r3 = p == 0 ? tl.q[c][3].x : (p == 1 ? tl.q[c][3].y : (p == 2 ? tl.q[c][3].z : tl.q[c][3].w));
                        // column 2p: the low halves of the four rows; column 2p + 1: the high halves
                        const uint2 be = make_uint2(__builtin_amdgcn_perm(r1, r0, 0x05040100u), __builtin_amdgcn_perm(r3, r2, 0x05040100u));
                        const uint2 bo = make_uint2(__builtin_amdgcn_perm(r1, r0, 0x07060302u), __builtin_amdgcn_perm(r3, r2, 0x07060302u));
                        const h16x4 fe = __builtin_bit_cast(h16x4, be), fo = __builtin_bit_cast(h16x4, bo);
                        acc[c][2 * p] = __builtin_amdgcn_mfma_f32_16x16x16f16(hhi, fe, acc[c][2 * p], 0, 0, 0);
                        acc[c][2 * p] = __builtin_amdgcn_mfma_f32_16x16x16f16(hlo, fe, acc[c][2 * p], 0, 0, 0);
                        acc[c][2 * p + 1] = __builtin_amdgcn_mfma_f32_16x16x16f16(hhi, fo, acc[c][2 * p + 1], 0, 0, 0);
                        acc[c][2 * p + 1] = __builtin_amdgcn_mfma_f32_16x16x16f16(hlo, fo, acc[c][2 * p + 1], 0, 0, 0);
                    }
                }
            };
            // two tiles on their way while one is computed
            DownTile t0, t1, t2;
            load_tile(t0, 0);
            load_tile(t1, 1);
#pragma unroll 1
            for (int t = 0; t < ntiles; t += 3) {
                load_tile(t2, t + 2);
                compute_tile(t0);
                load_tile(t0, t + 3);
                if (t + 1 < ntiles) compute_tile(t1);
                load_tile(t1, t + 4);
                if (t + 2 < ntiles) compute_tile(t2);
            }
        }
    }
    // lane (l16, g) holds Y[token 4g + i][column col0 + 128 c + 8 l16 + j]
    if (!wave_live) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = 4 * g + i;
        if (n >= n_tok) continue;
        const int task = grp->task[n];
        float* out = a.partial + ((size_t)task * a.nblk_down + blockIdx.x) * d + col0 + 8 * l16;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if (c >= ncw) break;
            float4* o4 = reinterpret_cast<float4*>(out + 128 * c);
            o4[0] = make_float4(acc[c][0][i], acc[c][1][i], acc[c][2][i], acc[c][3][i]);
            o4[1] = make_float4(acc[c][4][i], acc[c][5][i], acc[c][6][i], acc[c][7][i]);
        }
    }
}


// ---------------------------------------------------------------------------------------------------------------
// Steps 4-5 of a group in ONE kernel, the rows staged through LDS: workgroup = (group, block of channels), one wave per
// token of the group (16 waves).  The [gate | down] chunks of the block's union rows travel from HBM straight into a
// ring in LDS (global_load_lds_dwordx4: whole chunks, 1 KiB per wave instruction, no register is held in flight),
// two stages of 64 KiB: while one stage is consumed the next one lands.  A wave keeps its token's activations and its
// 4 d bytes of accumulators in registers, looks at the rows of the stage that ITS token selected, and for each of them
// reads the chunk from LDS: gate . x on packed dot products, SiLU, times v and the combine weight, then y += h * down.
// Every row is read from HBM once per group; the arithmetic is that of the (token, row) pairs that were selected, as in
// the one-token kernels, and each token's sum is formed in ascending channel order (reproducible bit for bit).
// The ring is written by the DMA loads and read with hand-placed ds_read_b128 (the compiler would make every LDS read
// wait for all loads in flight): a stage is read only after every wave has waited for its own loads of that stage and
// passed a barrier, and is requested again only after a barrier behind its last read.
// ---------------------------------------------------------------------------------------------------------------
constexpr int kFusedUnionWaves = 16;
constexpr int kStageBytes = 64 * 1024;

__device__ __forceinline__ void dma1k_to_lds(const void* src_lane, void* lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const FLOE_GLOBAL void*)src_lane, (__attribute__((address_space(3))) void*)lds_wave_base, 16,
                                     0, 0);
}
// two 16-byte reads of this lane at lds_addr and lds_addr + 1 KiB, complete on return
__device__ __forceinline__ void lds_read2x16(uint32_t lds_addr, u32x4& q0, u32x4& q1) {
    asm volatile(
        "ds_read_b128 %0, %2\n\t"
        "ds_read_b128 %1, %2 offset:1024\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(q0), "=&v"(q1)
        : "v"(lds_addr)
        : "memory");
}
__device__ __forceinline__ void lds_read1x16(uint32_t lds_addr, u32x4& q0) {
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(q0) : "v"(lds_addr) : "memory");
}
// A list word read from LDS, complete on return.  Inside the ring loop every LDS and memory read is issued by hand:
// for reads that the compiler places itself it charges a wait for ALL loads in flight (it cannot tell the ring's
// direct-to-LDS loads from anything else), which would serialise the ring.
__device__ __forceinline__ uint32_t lds_read_word(uint32_t lds_addr) {
    uint32_t r;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(r) : "v"(lds_addr) : "memory");
    return r;
}
// A 4-byte load whose arrival the caller waits for itself (wait_vm_le) before settle() hands the value out.
__device__ __forceinline__ void gload4_unwaited(const void* p, uint32_t& r) {
    asm volatile("global_load_dword %0, %1, off" : "=&v"(r) : "v"(p) : "memory");
}
__device__ __forceinline__ void settle(uint32_t& r) { asm volatile("" : "+v"(r) : : "memory"); }

template <int N>
__device__ __forceinline__ void wait_vm_le() {  // s_waitcnt vmcnt(N) only (gfx9 encoding: bits 3:0 and 15:14)
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <int NV>  // d = 512 * NV <= 4096
__global__ __launch_bounds__(kFusedUnionWaves * 64) void union_fused_kernel(UnionArgs a) {
    constexpr int d = 512 * NV;
    constexpr int kChunk = 4 * d;                       // bytes of a [gate | down] chunk
    constexpr int R = kStageBytes / kChunk;             // rows per stage (4 at d = 4096)
    constexpr int kPieces = kStageBytes / 1024;         // 1 KiB pieces per stage
    constexpr int kPpw = kPieces / kFusedUnionWaves;    // pieces a wave requests per stage (4)
    constexpr int kPpr = kChunk / 1024;                 // pieces per row
    static_assert(kPieces % kFusedUnionWaves == 0 && R >= 1, "stage split");
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char* ring = lds;                                              // [2][kStageBytes]
    int* lrow = reinterpret_cast<int*>(lds + 2 * kStageBytes);              // [cap]
    uint32_t* lbits = reinterpret_cast<uint32_t*>(lrow + a.cap);            // [cap]
    __shared__ int s_task[16];
    __shared__ float s_w[16];
    __shared__ int s_count;

    if ((int)blockIdx.y >= a.n_groups[0]) return;
    const TokenGroup* grp = a.groups + blockIdx.y;
    const int n_tok = grp->n;
    const DevExpert e = a.table[grp->expert];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int blk = blockIdx.x;
    union_tasks(a, grp, n_tok, s_task, s_w);
    const int count = union_list(a, grp, n_tok, blk, lrow, lbits, s_task, &s_count);
    const bool tok_wave = wave < n_tok;  // this wave owns a token (the others only help to request the rows)
    const int task = s_task[tok_wave ? wave : 0];
    const float w = s_w[tok_wave ? wave : 0];
    const float* vt = a.v + (size_t)task * a.f;

    // this token's activations: piece c of the lane = x[(c * 64 + lane) * 8 ..], the layout of a gate column in a chunk
    uint4 xr[NV];
    {
        const uint4* xp = reinterpret_cast<const uint4*>(a.x + (size_t)(task / a.slots) * d);
#pragma unroll
        for (int c = 0; c < NV; ++c) xr[c] = gload16(xp + c * kWave + lane);
    }
    float acc[8 * NV];
#pragma unroll
    for (int i = 0; i < 8 * NV; ++i) acc[i] = 0.0f;
    wait_vm_le<0>();  // x has arrived: inside the loop no wait may be charged to it (it would wait for the ring's loads)

    const int nstages = (count + R - 1) / R;
    const unsigned char* gd8 = reinterpret_cast<const unsigned char*>(e.gd);
    const uint32_t lrow_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)lrow;
    const uint32_t lbits_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)lbits;
    auto row_at = [&](int k) { return (int)lds_read_word(lrow_addr + 4 * (uint32_t)min(k, count - 1)); };
    // request stage s: piece p = wave * kPpw + j of the stage is 1 KiB number (p % kPpr) of row (p / kPpr); rows past
    // the end of the list repeat the last row (cache hits that nobody reads), so the request count never varies
    auto request = [&](int s) {
        unsigned char* dst = ring + (s & 1) * kStageBytes;
#pragma unroll
        for (int j = 0; j < kPpw; ++j) {
            const int p = wave * kPpw + j;
            const unsigned char* src = gd8 + (size_t)row_at(s * R + p / kPpr) * kChunk + (p % kPpr) * 1024 + lane * 16;
            dma1k_to_lds(src, dst + p * 1024);
        }
    };
    const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring + lane * 16;
    if (nstages > 0) request(0);
    for (int s = 0; s < nstages; ++s) {
        // v of the stage's rows for this wave's token: lane r fetches row r's, handed out by readlane after the wait
        uint32_t vraw;
        gload4_unwaited(vt + row_at(s * R + (lane < R ? lane : 0)), vraw);
        if (s + 1 < nstages) {
            request(s + 1);
            wait_vm_le<kPpw>();  // everything but the kPpw requests just made: stage s and v have arrived
        } else {
            wait_vm_le<0>();
        }
        settle(vraw);
        __builtin_amdgcn_s_barrier();  // ... for every wave
        if (tok_wave) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int k = s * R + r;
                if (k >= count) break;                                                     // wave-uniform
                const uint32_t bits = __builtin_amdgcn_readfirstlane(lds_read_word(lbits_addr + 4 * (uint32_t)k));
                if (!((bits >> wave) & 1u)) continue;      // wave-uniform: the token did not select this row
                const uint32_t base = ring_addr + (s & 1) * kStageBytes + r * kChunk;
                float g = 0.0f;
#pragma unroll
                for (int c0 = 0; c0 < NV; c0 += 2) {
                    u32x4 q[2];
                    if (c0 + 1 < NV) lds_read2x16(base + c0 * 1024, q[0], q[1]);
                    else lds_read1x16(base + c0 * 1024, q[0]);
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        if (c0 + c >= NV) break;
                        g = dot2(xr[c0 + c].x, q[c].x, g);
                        g = dot2(xr[c0 + c].y, q[c].y, g);
                        g = dot2(xr[c0 + c].z, q[c].z, g);
                        g = dot2(xr[c0 + c].w, q[c].w, g);
                    }
                }
                g = wave_allreduce_sum(g);
                const float vv = __builtin_bit_cast(float, __builtin_amdgcn_readlane((int)vraw, r));
                const float h = silu(g) * vv * w;
#pragma unroll
                for (int c0 = 0; c0 < NV; c0 += 2) {
                    u32x4 q[2];
                    if (c0 + 1 < NV) lds_read2x16(base + 2 * d + c0 * 1024, q[0], q[1]);
                    else lds_read1x16(base + 2 * d + c0 * 1024, q[0]);
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        if (c0 + c >= NV) break;
                        const uint32_t wds[4] = {q[c].x, q[c].y, q[c].z, q[c].w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const h16x2 pr = as_h2(wds[i]);
                            acc[(c0 + c) * 8 + 2 * i + 0] = fmaf(h, (float)pr.x, acc[(c0 + c) * 8 + 2 * i + 0]);
                            acc[(c0 + c) * 8 + 2 * i + 1] = fmaf(h, (float)pr.y, acc[(c0 + c) * 8 + 2 * i + 1]);
                        }
                    }
                }
            }
        }
        __builtin_amdgcn_s_barrier();  // every wave is done with stage s: its half of the ring may be requested again
    }
    // lane owns columns [(c * 64 + lane) * 8, + 8)
    if (tok_wave) {
        float* out = a.partial + ((size_t)task * a.nblk_down + blk) * d;
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            float4* o4 = reinterpret_cast<float4*>(out + (size_t)(c * kWave + lane) * 8);
            o4[0] = make_float4(acc[c * 8 + 0], acc[c * 8 + 1], acc[c * 8 + 2], acc[c * 8 + 3]);
            o4[1] = make_float4(acc[c * 8 + 4], acc[c * 8 + 5], acc[c * 8 + 6], acc[c * 8 + 7]);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------------------
// Which kernels run steps 4-5 of a decode batch (floe_tuning): 0 = chosen per call (below), 1 = matrix cores
// (gate_union_kernel + down_union_kernel), 2 = rows staged through an LDS ring (union_fused_kernel), 3 = the one-token
// kernels launched in expert order (rows that several tokens selected are shared through the L2).  Process-wide:
// workspace sizes depend on it, so it must not change between a size query and the call that uses the workspace.
static std::atomic<int> g_union_mode{0};
int union_mode() { return g_union_mode.load(std::memory_order_relaxed); }
void set_union_mode(int m) { g_union_mode.store(m >= 0 && m <= 3 ? m : 0, std::memory_order_relaxed); }
// Measured (8 experts, d = 4096, f = 14336, 90 %): the matrix-core pair overtakes the one-token kernels once an expert
// sees about a dozen tokens (its union is then most of the matrix and every row serves several tokens).
int union_kernels_for(int n_all, int n_tasks) {
    const int m = union_mode();
    if (m != 0) return m;
    return (long long)n_tasks >= 12ll * n_all ? 1 : 3;
}

// Expected number of token groups when n_tasks (token, slot) pairs fall on n_all experts uniformly: per expert
// E[ceil(X / chunk)] = sum over k >= 0 of P(X > k * chunk), X binomial, by its normal approximation.
static double expected_groups(int n_all, int n_tasks, int chunk) {
    const double pr = 1.0 / n_all, mu = n_tasks * pr, sd = sqrt(n_tasks * pr * (1.0 - pr)) + 1e-9;
    double per = 0.0;
    for (int k = 0; k * chunk < n_tasks; ++k) per += 0.5 * erfc(((double)k * chunk + 0.5 - mu) / (sd * 1.4142135623730951));
    return per * n_all;
}

UnionPlan union_plan(int d, int f, int n_tasks, int n_all, int chunk) {
    UnionPlan p{};
    const int nwords = mask_words_per_task(f);
    p.max_groups = mfma_max_groups(n_all, n_tasks);
    const int kernels = union_kernels_for(n_all, n_tasks);
    p.matrix_cores = kernels == 1;
    p.fused = kernels == 2;
    // Gate workgroups hold the group's activations in LDS, one per compute unit: a launch of a little less than one
    // workgroup per compute unit for the groups to be expected runs in one round (a few more and it takes two).
    const double est = expected_groups(n_all, n_tasks, chunk);
    int nb = (int)(0.95 * num_cus() / (est > 1.0 ? est : 1.0));
    nb = nb < 1 ? 1 : (nb > nwords ? nwords : nb);
    // at least two tiles of work per wave where the block is long enough: 16 rows x 8 waves x 2 = 256 channels = 8 words
    const int by_len = (nwords + 7) / 8;
    nb = nb > by_len ? by_len : nb;
    nb = nb < 1 ? 1 : nb;
    if (p.matrix_cores) {
        // down blocks: a divisor of the gate blocks, about half as many (fewer partial results to add up afterwards)
        p.nblk_down = nb >= 2 ? nb / 2 : 1;
        p.nblk_gate = p.nblk_down * (nb / p.nblk_down);
    } else {
        p.nblk_down = p.nblk_gate = nb;  // one kernel: the block that gathers the rows also stores the partial results
    }
    const int per = (nwords + p.nblk_gate - 1) / p.nblk_gate;
    p.cap = ((per * 32 + 15) / 16) * 16;
    p.nt = chunk <= 8 ? 8 : 16;
    return p;
}

size_t union_lds_bytes(int d, const UnionPlan& p) {
    if (p.fused) return (size_t)2 * kStageBytes + (size_t)p.cap * 8;
    return (size_t)p.nt * (d * 2 + 16) + (size_t)p.cap * 8;
}

template <int NV>
static hipError_t launch_gate_nv(const UnionArgs& a, const UnionPlan& p, hipStream_t stream) {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> attr_bytes[kMaxDevices];  // largest dynamic LDS size enabled so far, per device
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    const int lds = (int)union_lds_bytes(512 * NV, p);
    if (attr_bytes[dev].load(std::memory_order_acquire) < lds) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&gate_union_kernel<NV>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (rc != hipSuccess) return rc;
        attr_bytes[dev].store(lds, std::memory_order_release);
    }
    gate_union_kernel<NV><<<dim3(p.nblk_gate, p.max_groups), dim3(kGateWaves * 64), lds, stream>>>(a);
    return hipGetLastError();
}

bool union_shape_ok(int d, int f, const UnionPlan& p) {
    // (the ring kernel keeps a token's 4 d bytes of accumulators in one wave's registers: d <= 4096)
    return mask_words_per_task(f) <= 2048 && union_lds_bytes(d, p) <= 150 * 1024 && (p.matrix_cores || d <= 4096);
}

template <int NV>
static hipError_t launch_fused_nv(const UnionArgs& a, const UnionPlan& p, hipStream_t stream) {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> attr_bytes[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    const int lds = (int)union_lds_bytes(512 * NV, p);
    if (attr_bytes[dev].load(std::memory_order_acquire) < lds) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&union_fused_kernel<NV>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (rc != hipSuccess) return rc;
        attr_bytes[dev].store(lds, std::memory_order_release);
    }
    union_fused_kernel<NV><<<dim3(p.nblk_gate, p.max_groups), dim3(kFusedUnionWaves * 64), lds, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_gate_down_union(const UnionArgs& a, const UnionPlan& p, int d, hipStream_t stream) {
    hipError_t rc;
    if (p.fused) {
        switch (d / 512) {
#define FLOE_NV_CASE(N) case N: return launch_fused_nv<N>(a, p, stream);
            FLOE_NV_CASE(1) FLOE_NV_CASE(2) FLOE_NV_CASE(3) FLOE_NV_CASE(4) FLOE_NV_CASE(5) FLOE_NV_CASE(6)
            FLOE_NV_CASE(7) FLOE_NV_CASE(8)
#undef FLOE_NV_CASE
            default: return hipErrorInvalidValue;
        }
    }
    switch (d / 512) {
#define FLOE_NV_CASE(N) case N: rc = launch_gate_nv<N>(a, p, stream); break;
        FLOE_NV_CASE(1) FLOE_NV_CASE(2) FLOE_NV_CASE(3) FLOE_NV_CASE(4) FLOE_NV_CASE(5) FLOE_NV_CASE(6)
        FLOE_NV_CASE(7) FLOE_NV_CASE(8) FLOE_NV_CASE(9) FLOE_NV_CASE(10) FLOE_NV_CASE(11) FLOE_NV_CASE(12)
        FLOE_NV_CASE(13) FLOE_NV_CASE(14) FLOE_NV_CASE(15) FLOE_NV_CASE(16)
#undef FLOE_NV_CASE
        default: return hipErrorInvalidValue;
    }
    if (rc != hipSuccess) return rc;
    const int ncol = (d + kDownColsPerWg - 1) / kDownColsPerWg;
    down_union_kernel<<<dim3(p.nblk_down, p.max_groups, ncol), dim3(kDownWaves * 64), (size_t)p.cap * 4, stream>>>(a, d);
    return hipGetLastError();
}

}  // namespace floe
