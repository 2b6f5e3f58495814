// S2 for several tokens at once (decode batches): V = X . W_up^Q with the tokens that were routed to the
// same expert sharing ONE pass over that expert's codes (Alg. 1 line 2; the paper itself is batch-1, each
// token keeps its own threshold, mask and result).  Here the contraction is dense and tall-skinny
// (up to 16 tokens x d) x (d x f), so it goes to the matrix cores:
//
//   v_mfma_f32_16x16x32_f16:  C[16 tokens][16 channels] += A[16 tokens][32 k] * B[32 k][16 channels]
//
// * B (weights) never becomes a number on the vector ALU.  A lane (channel c = lane % 16, quarter
//   g = lane / 16) loads the 16 codes of its quarter of a 64-code unit (one dword for INT2, two for INT4).
//   A code field that sits at bits [p, p+b) of a 16-bit half, ANDed out and left in place, IS the fp16
//   subnormal q * 2^(p-24) (the matrix cores honour fp16 subnormals), so one AND per register builds
//   two weights, with no offset to remove afterwards.
// * A (activations) is prepared once per workgroup in LDS in exactly the slot order the extraction
//   produces, pre-multiplied by 2^(pmax - p) so that every product carries the same 2^(pmax-24), and by a
//   per-token power of two that keeps it finite in fp16.
// * Two MFMAs cover the 64 codes of a unit.  The result tile is scaled per quantization group,
//   acc += s * (2^k C - z * Xg), with the channel's (s, z) in the lane and the tokens' group sums Xg in
//   LDS.  A lane ends up holding v for one channel and four tokens; the comparison with each token's
//   threshold is a wave ballot whose 16-bit pieces are the mask bits the gate/down kernel compacts.
#include <atomic>

#include "floe_dev.h"
#include "launch.h"

namespace floe {

typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaThreads = 512;              // 8 waves

static std::atomic<int> g_grouped_gemv_mode{0};
int grouped_gemv_mode() { return g_grouped_gemv_mode.load(std::memory_order_relaxed); }
void set_grouped_gemv_mode(int m) { g_grouped_gemv_mode.store(m >= 0 && m <= 2 ? m : 0, std::memory_order_relaxed); }

// How the 64 codes of a unit are dealt to the four lane quarters g and the two MFMAs j.
//  kLaneWords           code words a lane loads per unit
//  word(k, g)           index (inside the unit) of the lane's k-th word
//  code(j, g, s)        code index (0..63 inside the unit) that slot s of MFMA j holds in quarter g
//  pos(j, s)            bit position of that code's field inside its 16-bit half
//  kPmax                every product carries 2^(kPmax - 24)
// With one quantization group per unit (G32 = false) any dealing works because both MFMAs are summed
// before scaling; with groups of 32 MFMA j must cover exactly the codes 32j .. 32j+31.
template <int BITS, bool G32> struct MfmaTraits;
template <> struct MfmaTraits<2, false> {  // quarter g owns word g (codes 16g .. 16g+15)
    static constexpr int kLaneWords = 1;
    static constexpr int kPmax = 8;
    __device__ static constexpr int word(int k, int g) { (void)k; return g; }
    __device__ static constexpr int code(int j, int g, int s) {
        constexpr int t[2][8] = {{0, 8, 1, 9, 2, 10, 3, 11}, {4, 12, 5, 13, 6, 14, 7, 15}};
        return 16 * g + t[j][s];
    }
    __device__ static constexpr int pos(int j, int s) {
        constexpr int t[2][8] = {{4, 4, 6, 6, 4, 4, 6, 6}, {8, 8, 4, 4, 6, 6, 8, 8}};
        return t[j][s];
    }
};
template <bool G32> struct MfmaTraits<4, G32> {  // MFMA j reads word 4j + g: it covers codes 32j .. 32j+31
    static constexpr int kLaneWords = 2;
    static constexpr int kPmax = 6;
    __device__ static constexpr int word(int k, int g) { return 4 * k + g; }
    __device__ static constexpr int code(int j, int g, int s) {
        constexpr int t[8] = {0, 4, 1, 5, 2, 6, 3, 7};
        return 32 * j + 8 * g + t[s];
    }
    __device__ static constexpr int pos(int j, int s) {
        constexpr int t[8] = {4, 4, 4, 4, 2, 2, 6, 6};
        (void)j;
        return t[s];
    }
};

// INT3: the 32 codes of a half unit are 96 contiguous bits; quarter g owns the 24 bits [24g, 24g + 24) of them, which
// lie in words a, a + 1 of the half unit with a = g / 2.  A lane loads those two words itself (kOwnWords) and shifts
// its field down; codes 0..3 of the field stay in the low 16-bit half, codes 4..7 move to the high half.
template <bool G32> struct MfmaTraits<3, G32> {
    static constexpr int kLaneWords = 4;  // two words for each of the two MFMAs
    static constexpr int kPmax = 6;
    __device__ static constexpr int word(int k, int g) { return 3 * (k >> 1) + (g >> 1) + (k & 1); }
    __device__ static constexpr int code(int j, int g, int s) {
        constexpr int t[8] = {0, 4, 1, 5, 2, 6, 3, 7};
        return 32 * j + 8 * g + t[s];
    }
    __device__ static constexpr int pos(int j, int s) {
        constexpr int t[8] = {0, 0, 3, 3, 6, 6, 6, 6};
        (void)j;
        return t[s];
    }
};

// the 4 registers (8 fp16 subnormals) of MFMA j from the lane's code words
template <int BITS, bool G32>
__device__ __forceinline__ void weight_frag(const uint32_t* w, int j, int g, uint32_t (&r)[4]) {
    if (BITS == 3) {
        // w[2j], w[2j+1]: the two words that hold the quarter's 24 bits, at bit 24g - 32(g/2) of the pair
        const uint64_t pair = ((uint64_t)w[2 * j + 1] << 32) | w[2 * j];
        const uint32_t c24 = (uint32_t)(pair >> (24 * g - 32 * (g >> 1)));
        const uint32_t t = (c24 & 0x00000FFFu) | ((c24 << 4) & 0x0FFF0000u);
        r[0] = t & 0x00070007u;         // codes (0, 4) at bits [0,3)
        r[1] = t & 0x00380038u;         // codes (1, 5) at bits [3,6)
        r[2] = t & 0x01C001C0u;         // codes (2, 6) at bits [6,9)
        r[3] = (t >> 3) & 0x01C001C0u;  // codes (3, 7) from bits [9,12) to [6,9)
    } else if (BITS == 2 && !G32) {
        const uint32_t W = w[0], a = W << 4, b = W >> 6;
        if (j == 0) {
            r[0] = a & 0x00300030u;  // codes (0, 8)  at bits [4,6)
            r[1] = a & 0x00C000C0u;  // codes (1, 9)  at bits [6,8)
            r[2] = W & 0x00300030u;  // codes (2, 10) at bits [4,6)
            r[3] = W & 0x00C000C0u;  // codes (3, 11) at bits [6,8)
        } else {
            r[0] = W & 0x03000300u;  // codes (4, 12) at bits [8,10)
            r[1] = b & 0x00300030u;  // codes (5, 13) at bits [4,6)
            r[2] = b & 0x00C000C0u;  // codes (6, 14) at bits [6,8)
            r[3] = b & 0x03000300u;  // codes (7, 15) at bits [8,10)
        }
    } else {
        const uint32_t W = w[j], a = W << 4, b = W >> 6;
        r[0] = a & 0x00F000F0u;      // codes (0, 4) at bits [4,8)
        r[1] = W & 0x00F000F0u;      // codes (1, 5) at bits [4,8)
        r[2] = b & 0x003C003Cu;      // codes (2, 6) at bits [2,6)
        r[3] = b & 0x03C003C0u;      // codes (3, 7) at bits [6,10)
    }
}

__device__ __forceinline__ h16x8 as_h8(const uint32_t (&r)[4]) {
    uint4 q = make_uint4(r[0], r[1], r[2], r[3]);
    return __builtin_bit_cast(h16x8, q);
}

template <int BITS, int UPC, bool G32, int NTPAD, int TILES>
__global__ __launch_bounds__(kMfmaThreads, BITS == 3 ? 4 : 1) void up_gemv_mfma_kernel(const DevExpert* __restrict__ table,
                                                                     const TokenGroup* __restrict__ groups,
                                                                     const int32_t* __restrict__ n_groups,
                                                                     const h16* __restrict__ x, int slots,
                                                                     float* __restrict__ v,
                                                                     const float* __restrict__ task_tau,
                                                                     uint32_t* __restrict__ mask_words, int f) {
    using Tr = MfmaTraits<BITS, G32>;
    constexpr int d = UPC * 64;
    constexpr int LW = Tr::kLaneWords;
    constexpr int kCw = BITS * 2;               // code words per unit (64 codes)
    constexpr int LWQ = kCw / 4;                // 128-bit vectors per unit
    constexpr bool kOwnWords = BITS == 3;       // every lane loads the words of its own quarter (no exchange)
    constexpr int GPU_ = G32 ? 2 : 1;           // quantization groups per unit
    constexpr int kGroupsPerRow = UPC * GPU_;   // scale / zero entries per channel
    constexpr float kScaleBack = (float)(1 << (24 - Tr::kPmax));
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint4* xfrag = reinterpret_cast<uint4*>(lds_raw);                         // [UPC][2][4][NTPAD]
    float* xg = reinterpret_cast<float*>(xfrag + (size_t)UPC * 8 * NTPAD);   // [UPC * GPU_][NTPAD]
    __shared__ float tok_inv_p[16];
    __shared__ float tok_tau[16];
    __shared__ int tok_task[16];
    __shared__ int tok_down[16];
    __shared__ unsigned tok_amax[16];

    if ((int)blockIdx.y >= n_groups[0]) return;  // the grid is sized for the worst case
    const TokenGroup* grp = groups + blockIdx.y;  // read in place: indexing a register copy would spill
    const DevExpert e = table[grp->expert];
    const int n_tok = grp->n;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int c = lane & 15, g = lane >> 4;

    FLOE_TL(0);
    // ---- activations.  One thread per (unit, token) keeps the unit's 64 activations (128 contiguous
    // bytes) in registers across three steps: (1) the token's largest magnitude, met in LDS with an
    // integer max on the bit patterns, gives a power of two that keeps 16 * |x'| finite in fp16;
    // (2) the scaled activations go to LDS as the fragments the MFMAs read: entry (U, j, g, n) holds the
    // 8 values that meet MFMA j of unit U in lane quarter g for token n, in slot order, each times
    // 2^(pmax - p); all offsets are compile-time constants; (3) the group sums of x' go beside them.
    constexpr int kEnt = (UPC * NTPAD + kMfmaThreads - 1) / kMfmaThreads;  // entries per thread
    if (tid < 16) {
        tok_amax[tid] = 0u;
        const bool livetok = tid < n_tok && tid < NTPAD;
        tok_task[tid] = livetok ? grp->task[tid] : -1;
        tok_tau[tid] = (livetok && task_tau) ? task_tau[grp->task[tid]] : 0.0f;
    }
    __syncthreads();
    uint4 xq[kEnt][8];
#pragma unroll
    for (int en = 0; en < kEnt; ++en) {
        const int idx = tid + en * kMfmaThreads;
        const int n = idx % NTPAD, U = idx / NTPAD;
        float amax = 0.0f;
        if (idx < UPC * NTPAD && n < n_tok) {
            const int t = tok_task[n] / slots;
            const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)t * d + U * 64);
#pragma unroll
            for (int r = 0; r < 8; ++r) xq[en][r] = xr[r];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const uint32_t wds[4] = {xq[en][r].x, xq[en][r].y, xq[en][r].z, xq[en][r].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const h16x2 p = as_h2(wds[k]);
                    amax = fmaxf(amax, fmaxf(fabsf((float)p.x), fabsf((float)p.y)));
                }
            }
            atomicMax(&tok_amax[n], __builtin_bit_cast(unsigned, amax));  // non-negative floats order like integers
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r) xq[en][r] = make_uint4(0u, 0u, 0u, 0u);
        }
    }
    __syncthreads();
    if (tid < 16) {
        const float amax = __builtin_bit_cast(float, tok_amax[tid]);
        const int down = (amax >= 512.0f && amax < 3.0e38f) ? ilogbf(amax) - 8 : 0;  // |x'| < 512
        tok_down[tid] = down;
        tok_inv_p[tid] = ldexpf(1.0f, down) * kScaleBack;  // undoes the token's pre-scaling and the 2^(pmax - 24) of the products
    }
    __syncthreads();
    FLOE_TL(1);
#pragma unroll
    for (int en = 0; en < kEnt; ++en) {
        const int idx = tid + en * kMfmaThreads;
        if (idx >= UPC * NTPAD) continue;
        const int n = idx % NTPAD, U = idx / NTPAD;
        unsigned char* ubase = lds_raw + (size_t)U * (8 * NTPAD * 16) + n * 16;
        const h16 ps = (h16)ldexpf(1.0f, -tok_down[n]);
        const h16x2 ps2 = {ps, ps};
        uint32_t xv[32];  // (x'[2i], x'[2i+1])
        float gsum[2] = {0.0f, 0.0f};
        const h16x2 ones = {(h16)1.0f, (h16)1.0f};
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint32_t wds[4] = {xq[en][r].x, xq[en][r].y, xq[en][r].z, xq[en][r].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const h16x2 p = as_h2(wds[k]) * ps2;
                xv[4 * r + k] = as_u32(p);
                gsum[G32 ? (r >> 2) : 0] = __builtin_amdgcn_fdot2(p, ones, gsum[G32 ? (r >> 2) : 0], false);
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq)
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) {
                    const int lo = Tr::code(j, gq, 2 * pr), hi = Tr::code(j, gq, 2 * pr + 1);
                    const uint32_t wl = xv[lo >> 1], wh = xv[hi >> 1];
                    const uint32_t l16 = (lo & 1) ? (wl >> 16) : (wl & 0xFFFFu);
                    const uint32_t h16b = (hi & 1) ? (wh & 0xFFFF0000u) : (wh << 16);
                    const h16x2 mul = {(h16)(float)(1 << (Tr::kPmax - Tr::pos(j, 2 * pr))),
                                       (h16)(float)(1 << (Tr::kPmax - Tr::pos(j, 2 * pr + 1)))};
                    const h16x2 val = as_h2(l16 | h16b) * mul;
                    *reinterpret_cast<uint32_t*>(ubase + ((j * 4 + gq) * NTPAD) * 16 + 4 * pr) = as_u32(val);
                }
#pragma unroll
        // (times 2^(pmax - 24): the matrix products carry that factor, and the zero-point term is subtracted from them
        // before the scale is applied)
        for (int q2 = 0; q2 < GPU_; ++q2) xg[(size_t)(U * GPU_ + q2) * NTPAD + n] = gsum[q2] * (1.0f / kScaleBack);
    }
    __syncthreads();

    FLOE_TL(2);
    // ---- main loop: this wave owns TILES tiles of 16 channels, all UPC units, in blocks of 8 units.
    // Loads are line-wide: quarter g of a channel's four lanes fetches units 8B+2g and 8B+2g+1 whole
    // (the four quarters together read contiguous 128 / 256 bytes), and a 4x4 transpose across the lane
    // quarters (v_permlane32_swap + v_permlane16_swap) hands every quarter ITS word of each unit.
    // Scales and zeros are fetched the same way (quarter g holds those of block 4Q+g) and passed to the
    // other quarters with ds_bpermute when their block comes up.
    // The workgroup walks the channel blocks blockIdx.x, blockIdx.x + gridDim.x, ...: the activation fragments above are
    // prepared once and serve all of them (with one workgroup per block their preparation was a third of the run time).
    const int n_cblocks = (f + 8 * 16 * TILES - 1) / (8 * 16 * TILES);
    for (int cb = blockIdx.x; cb < n_cblocks; cb += gridDim.x) {
    const int ch0 = (cb * 8 + wave) * (16 * TILES);
    // uniform base pointers plus 32-bit per-lane byte offsets (f <= 2^20 rows of <= 2 KiB)
    const char* cbase = reinterpret_cast<const char*>(e.codes);
    const char* sbase = reinterpret_cast<const char*>(e.scale);
    const char* zbase = reinterpret_cast<const char*>(e.zero);
    constexpr int kBlk = 8;                    // units per block
    constexpr int NB = UPC / kBlk;             // blocks per channel (2, 4 or 8)
    constexpr int NSB = (NB + 3) / 4;          // super-blocks of 4 blocks (meta registers)
    constexpr int kRaw = kOwnWords ? 1 : 2 * LWQ;  // uint4 a lane loads per tile per block (its two units)
    constexpr int kOwn = kOwnWords ? 2 * kBlk : 1;  // own-words form: a word pair per unit and MFMA
    constexpr int kMetaRegs = 4 * GPU_;        // 32-bit registers holding a block's 8 * GPU_ fp16 scales
    uint32_t coff[TILES], moff[TILES];
    int chan[TILES];
#pragma unroll
    for (int tt = 0; tt < TILES; ++tt) {
        chan[tt] = ch0 + 16 * tt + c;
        const uint32_t chl = chan[tt] < f ? chan[tt] : f - 1;  // clamped lanes load valid memory, never store
        coff[tt] = chl * (UPC * kCw) * 4u + (kOwnWords ? (uint32_t)(g >> 1) * 4u : (uint32_t)(2 * g) * (kCw * 4u));
        moff[tt] = chl * kGroupsPerRow * 2u;
    }
    float acc[TILES][4];
#pragma unroll
    for (int tt = 0; tt < TILES; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[tt][i] = 0.0f;

    // scales / zeros of the whole channel, dealt to the quarters: quarter g keeps block 4Q+g
    uint32_t ms[TILES][NSB][kMetaRegs], mz[TILES][NSB][kMetaRegs];
#pragma unroll
    for (int tt = 0; tt < TILES; ++tt)
#pragma unroll
        for (int Q = 0; Q < NSB; ++Q) {
            const int blk = (4 * Q + g) < NB ? (4 * Q + g) : NB - 1;
            const uint32_t off = moff[tt] + (uint32_t)(blk * kBlk * GPU_) * 2u;
#pragma unroll
            for (int r4 = 0; r4 < GPU_; ++r4) {
                // (the expert's pointers come out of a table in memory: say that they are global, or every load is a flat
                // one, which the LDS wait counter tracks as well)
                const uint4 a = gload16(sbase + off + 16 * r4);
                const uint4 bq = gload16(zbase + off + 16 * r4);
                ms[tt][Q][4 * r4 + 0] = a.x; ms[tt][Q][4 * r4 + 1] = a.y; ms[tt][Q][4 * r4 + 2] = a.z; ms[tt][Q][4 * r4 + 3] = a.w;
                mz[tt][Q][4 * r4 + 0] = bq.x; mz[tt][Q][4 * r4 + 1] = bq.y; mz[tt][Q][4 * r4 + 2] = bq.z; mz[tt][Q][4 * r4 + 3] = bq.w;
            }
        }

    struct Block {
        uint4 raw[TILES][kRaw];
        uint32_t own[TILES][kOwn][2];
    };
    auto load_block = [&](Block& b, int blk) {
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt) {
            const char* pb = cbase + (coff[tt] + (uint32_t)blk * (kBlk * kCw * 4u));
            if constexpr (kOwnWords) {
#pragma unroll
                for (int r = 0; r < kOwn; ++r) {  // r = 2 * unit + MFMA: half units are 12 bytes apart
                    b.own[tt][r][0] = gload4(pb + 12 * r);
                    b.own[tt][r][1] = gload4(pb + 12 * r + 4);
                }
            } else {
#pragma unroll
                for (int r = 0; r < kRaw; ++r) b.raw[tt][r] = gload16(pb + 16 * r);
            }
        }
    };
    auto transpose4 = [](uint4& q) {  // across the four lane quarters: register k <- word g of quarter k's vector
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        u32x2 t;
        t = __builtin_amdgcn_permlane32_swap(q.x, q.z, false, false); q.x = t.x; q.z = t.y;
        t = __builtin_amdgcn_permlane32_swap(q.y, q.w, false, false); q.y = t.x; q.w = t.y;
        t = __builtin_amdgcn_permlane16_swap(q.x, q.y, false, false); q.x = t.x; q.y = t.y;
        t = __builtin_amdgcn_permlane16_swap(q.z, q.w, false, false); q.z = t.x; q.w = t.y;
    };
    auto compute_block = [&](Block& b, int blk) {
        // meta of this block lives in quarter (blk % 4) of super-block blk / 4
        const int src_lane4 = (16 * (blk & 3) + c) * 4;
        uint32_t bs[TILES][kMetaRegs], bz[TILES][kMetaRegs];
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt)
#pragma unroll
            for (int r = 0; r < kMetaRegs; ++r) {
                uint32_t sv = ms[tt][0][r], zv = mz[tt][0][r];
                if (NSB > 1 && blk >= 4) { sv = ms[tt][NSB - 1][r]; zv = mz[tt][NSB - 1][r]; }
                bs[tt][r] = (uint32_t)__builtin_amdgcn_ds_bpermute(src_lane4, (int)sv);
                bz[tt][r] = (uint32_t)__builtin_amdgcn_ds_bpermute(src_lane4, (int)zv);
            }
        if constexpr (!kOwnWords) {
#pragma unroll
            for (int tt = 0; tt < TILES; ++tt)
#pragma unroll
                for (int r = 0; r < kRaw; ++r) transpose4(b.raw[tt][r]);
        }
        // after the transposes: raw[tt][h * LWQ + w4] component k = word (4 * w4 + g) of unit 2k + h
#pragma unroll
        for (int uu = 0; uu < kBlk; ++uu) {
            const int U = blk * kBlk + uu;
            const int kq = uu >> 1, h = uu & 1;
            h16x8 xa[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                // token rows beyond NTPAD repeat earlier ones; their results are never stored
                const uint4 q = xfrag[((size_t)(U * 2 + j) * 4 + g) * NTPAD + (c & (NTPAD - 1))];
                xa[j] = __builtin_bit_cast(h16x8, q);
            }
            float xgv[GPU_][4];
#pragma unroll
            for (int q = 0; q < GPU_; ++q)
#pragma unroll
                for (int i = 0; i < 4; ++i) xgv[q][i] = xg[(size_t)(U * GPU_ + q) * NTPAD + ((4 * g + i) & (NTPAD - 1))];
#pragma unroll
            for (int tt = 0; tt < TILES; ++tt) {
                uint32_t w[LW];
                if constexpr (kOwnWords) {
                    w[0] = b.own[tt][2 * uu][0]; w[1] = b.own[tt][2 * uu][1];
                    w[2] = b.own[tt][2 * uu + 1][0]; w[3] = b.own[tt][2 * uu + 1][1];
                } else {
#pragma unroll
                    for (int k = 0; k < LW; ++k) {
                        const uint4 q = b.raw[tt][h * LWQ + (LWQ == 1 ? 0 : k)];
                        w[k] = kq == 0 ? q.x : (kq == 1 ? q.y : (kq == 2 ? q.z : q.w));
                    }
                }
                uint32_t r0[4], r1[4];
                weight_frag<BITS, G32>(w, 0, g, r0);
                weight_frag<BITS, G32>(w, 1, g, r1);
                const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
                // scale and zero stay halves: the multiply-adds below take them as such (mixed-precision FMA), which
                // saves the two conversions and two products per unit that fp32 copies of s and s*z cost
                auto half_of = [](const uint32_t (&m)[kMetaRegs], int k) -> h16 {
                    const h16x2 p = as_h2(m[k >> 1]);
                    return (k & 1) ? p.y : p.x;
                };
                if (G32) {  // each half unit is a quantization group of its own
                    const f32x4 c0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[0], as_h8(r0), zero4, 0, 0, 0);
                    const f32x4 c1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[1], as_h8(r1), zero4, 0, 0, 0);
                    const h16 s0 = half_of(bs[tt], 2 * uu), z0 = half_of(bz[tt], 2 * uu);
                    const h16 s1 = half_of(bs[tt], 2 * uu + 1), z1 = half_of(bz[tt], 2 * uu + 1);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float t0 = fmaf(-(float)z0, xgv[0][i], c0[i]);
                        const float t1 = fmaf(-(float)z1, xgv[GPU_ - 1][i], c1[i]);
                        acc[tt][i] = fmaf((float)s1, t1, fmaf((float)s0, t0, acc[tt][i]));
                    }
                } else {
                    f32x4 cc = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[0], as_h8(r0), zero4, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[1], as_h8(r1), cc, 0, 0, 0);
                    const h16 s_h = half_of(bs[tt], uu), z_h = half_of(bz[tt], uu);
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[tt][i] = fmaf((float)s_h, fmaf(-(float)z_h, xgv[0][i], cc[i]), acc[tt][i]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads of later units from being hoisted up here
        }
    };

    static_assert(NB % 2 == 0, "units per channel must be a multiple of 16");
    FLOE_TL(3);
    if constexpr (kOwnWords) {
        // one block at a time: sixteen waves per compute unit (128 registers each) cover the round trips instead
        Block b0;
#pragma unroll 1
        for (int blk = 0; blk < NB; ++blk) {
            load_block(b0, blk);
            compute_block(b0, blk);
        }
    } else {
        Block b0, b1;
        load_block(b0, 0);
        for (int blk = 0; blk < NB; blk += 2) {
            load_block(b1, blk + 1);
            compute_block(b0, blk);
            if (blk + 2 < NB) load_block(b0, blk + 2);
            compute_block(b1, blk + 1);
        }
    }

    FLOE_TL(4);
    // ---- results: lane (c, g) holds channel chan[tt] for tokens 4g .. 4g+3
    const int nwords = mask_words_per_task(f);
    uint16_t* mask16 = reinterpret_cast<uint16_t*>(mask_words);
    const int f_pad = nwords * 32;
#pragma unroll
    for (int tt = 0; tt < TILES; ++tt) {
        const int tile_base = ch0 + 16 * tt;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int n = 4 * g + i;
            const bool live = n < n_tok;
            const float val = acc[tt][i] * tok_inv_p[n & 15];  // (tok_inv_p carries 2^(24 - pmax) as well)
            const int task = tok_task[n & 15];
            if (live && chan[tt] < f) v[(size_t)task * f + chan[tt]] = val;
            const bool keep = live && chan[tt] < f && fabsf(val) > tok_tau[n & 15];
            const uint64_t m = __ballot(keep);
            if (mask16 && live && c == 0 && tile_base < f_pad)
                mask16[(size_t)task * nwords * 2 + (tile_base >> 4)] = (uint16_t)(m >> (16 * g));
        }
    }
    }  // channel blocks
}

// ---------------------------------------------------------------------------------------------------
// Grouping: for every expert the ascending list of tasks (token, slot) routed to it, cut into chunks of
// `chunk` tasks.  One workgroup of 16 waves, a thread per task.  Deterministic (ascending expert, ascending task).
// order (optional): all tasks in that same order, i.e. sorted by expert (see gate_down.hip: workgroups of tasks that
// share an expert are launched next to each other so that they share the rows they both selected in the L2).
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void group_tokens_kernel(const int32_t* __restrict__ task_expert, int n_tasks,
                                                            int n_all, int chunk, TokenGroup* __restrict__ groups,
                                                            int32_t* __restrict__ n_groups, int32_t* __restrict__ order) {
    // A thread per task, 1024 tasks (16 waves of 64) at a time.  A task's place in its expert's list is
    //   (tasks of that expert in earlier tiles) + (in earlier waves of this tile) + (in lower lanes of this wave),
    // the last found by ballots over the distinct experts of the wave.  Every wave then stores its 64 tasks with two
    // instructions; written expert by expert instead, the stores had one or two lanes each and their number (not the
    // arithmetic) set the kernel's time.
    constexpr int kWaves = 16;
    constexpr int kTile = kWaves * kWave;
    constexpr int kMaxExperts = 1024 + 64;  // 1024 routed + 64 shared
    __shared__ int first_group[kMaxExperts + 1];
    __shared__ int first_task[kMaxExperts + 1];  // tasks of the experts before this one (for `order`)
    __shared__ int count[kMaxExperts];           // tasks per expert; in pass 2 the tasks placed by earlier tiles
    __shared__ __align__(16) uint8_t in_wave[kWaves][kMaxExperts];  // tasks of an expert inside one wave's 64 tasks of the tile
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const unsigned long long below = (1ull << lane) - 1ull;
    auto expert_of = [&](int task) {
        const int e = task < n_tasks ? task_expert[task] : -1;
        return (unsigned)e < (unsigned)n_all ? e : -1;  // an id outside the table belongs to no group
    };
    const bool one_tile = n_tasks <= kTile;  // the common case: the expert read in pass 1 serves pass 2 as well
    // pass 1: tasks per expert
    for (int e = tid; e < n_all; e += kTile) count[e] = 0;
    __syncthreads();
    int mine = -1;
    for (int base = 0; base < n_tasks; base += kTile) {
        mine = expert_of(base + tid);
        if (mine >= 0) atomicAdd(&count[mine], 1);  // integer adds in LDS: the order does not matter
    }
    __syncthreads();
    for (int e = tid; e < n_all; e += kTile) first_group[e + 1] = (count[e] + chunk - 1) / chunk;
    __syncthreads();
    if (wave == 0) {  // prefix sums over the experts, 64 at a time
        int run_g = 0, run_t = 0;
        for (int e0 = 0; e0 < n_all; e0 += kWave) {
            const int e = e0 + lane;
            int sg = e < n_all ? first_group[e + 1] : 0;
            int st = e < n_all ? count[e] : 0;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int ug = __shfl_up(sg, o, kWave), ut = __shfl_up(st, o, kWave);
                if (lane >= o) { sg += ug; st += ut; }
            }
            if (e < n_all) {
                first_group[e + 1] = run_g + sg;
                first_task[e + 1] = run_t + st;
            }
            run_g += __shfl(sg, kWave - 1, kWave);
            run_t += __shfl(st, kWave - 1, kWave);
        }
        if (lane == 0) {
            first_group[0] = 0;
            first_task[0] = 0;
            n_groups[0] = run_g;
        }
    }
    __syncthreads();
    // group headers; count[] then becomes the number of tasks that earlier tiles placed
    for (int e = tid; e < n_all; e += kTile) {
        const int g0 = first_group[e], ng = first_group[e + 1] - g0, c = count[e];
        for (int g = 0; g < ng; ++g) {
            groups[g0 + g].expert = e;
            groups[g0 + g].n = min(chunk, c - g * chunk);
        }
        count[e] = 0;
    }
    // pass 2: the tasks, in ascending order, into their chunks
    for (int base = 0; base < n_tasks; base += kTile) {
        for (int i = tid; i < kWaves * kMaxExperts / 4; i += kTile) reinterpret_cast<uint32_t*>(&in_wave[0][0])[i] = 0u;
        __syncthreads();  // in_wave cleared (and, the first time, the headers' reads of count[] are over)
        if (!one_tile) mine = expert_of(base + tid);
        int rank = 0;
        {
            unsigned long long todo = __ballot(mine >= 0);
            while (todo) {  // once per distinct expert among the wave's tasks
                const int e = __shfl(mine, __ffsll((long long)todo) - 1, kWave);
                const bool match = mine == e;
                const unsigned long long m = __ballot(match);
                if (match) {
                    rank = __popcll(m & below);
                    if (rank == 0) in_wave[wave][e] = (uint8_t)__popcll(m);
                }
                todo &= ~m;
            }
        }
        __syncthreads();
        if (mine >= 0) {
            int pos = count[mine] + rank;
            for (int w = 0; w < wave; ++w) pos += in_wave[w][mine];
            const int task = base + tid;
            groups[first_group[mine] + pos / chunk].task[pos % chunk] = task;
            if (order) order[first_task[mine] + pos] = task;
        }
        if (!one_tile) {
            __syncthreads();  // every read of count[] for this tile is over
            for (int e = tid; e < n_all; e += kTile) {
                int c = count[e];
#pragma unroll
                for (int w = 0; w < kWaves; ++w) c += in_wave[w][e];
                count[e] = c;
            }
            // the next tile's first barrier orders these writes before its reads; its clearing of in_wave needs one more
            __syncthreads();
        }
    }
}

#ifdef FLOE_TIMELINE
extern "C" int floe_debug_set_timeline_mfma(unsigned long long* p) {
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_timeline), &p, sizeof(p));
}
#endif

hipError_t launch_group_tokens(const int32_t* task_expert, int n_tasks, int n_all, int chunk, TokenGroup* groups,
                               int32_t* n_groups, hipStream_t stream, int32_t* order) {
    group_tokens_kernel<<<dim3(1), dim3(1024), 0, stream>>>(task_expert, n_tasks, n_all, chunk, groups, n_groups, order);
    return hipGetLastError();
}

// codes, scales and zeros of the channels one workgroup covers per block (8 waves x TILES tiles of 16 channels)
template <int BITS, int UPC, bool G32, int TILES>
constexpr size_t ch_per_wg_bytes() {
    return (size_t)(8 * 16 * TILES) * ((size_t)UPC * BITS * 8 + (size_t)UPC * (G32 ? 2 : 1) * 4);
}

template <int BITS, int UPC, bool G32, int NTPAD>
static hipError_t launch_mfma_inst(int max_groups, hipStream_t stream, const DevExpert* table, const TokenGroup* groups,
                                   const int32_t* n_groups, const h16* x, int slots, float* v, const float* task_tau,
                                   uint32_t* mask_words, int f) {
    // channels per wave = 16 * TILES: code blocks are double-buffered and all scales / zeros sit in registers
    constexpr int TILES = ((BITS == 4 && G32) || BITS == 3) ? 1 : 2;
    constexpr size_t lds = (size_t)UPC * 8 * NTPAD * 16 + (size_t)UPC * (G32 ? 2 : 1) * NTPAD * 4;
    // the attribute belongs to the function on one device: set once per device, from whichever thread comes first
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> attr_set[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&up_gemv_mfma_kernel<BITS, UPC, G32, NTPAD, TILES>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (rc != hipSuccess) return rc;
        attr_set[dev].store(true, std::memory_order_release);
    }
    const int ch_per_wg = 8 * 16 * TILES;
    // about two workgroups per compute unit over the groups that can exist at once, each taking an equal number of
    // channel blocks
    const int n_cblocks = (f + ch_per_wg - 1) / ch_per_wg;
    const int est_groups = max_groups > 2 ? (3 * max_groups + 3) / 4 : 1;
    const int wg_per_cu = lds > 80 * 1024 ? 1 : 2;  // what the fragments in LDS leave room for
    int want = (wg_per_cu * num_cus() + est_groups - 1) / est_groups;
    want = want < 1 ? 1 : (want > n_cblocks ? n_cblocks : want);
    int per_wg = (n_cblocks + want - 1) / want;
    // Short blocks (small d and f): one per workgroup, so that there are more workgroups than the chip holds at once
    // and the fragments of the later ones are prepared while the earlier ones stream (measured at d = 2048, f = 1408,
    // INT3: 145 us per layer call against 157 us at T = 32, 293 against 318 us at T = 128; with the 328 KB blocks of
    // d = 4096 fewer, longer workgroups stay faster).
    constexpr size_t block_bytes = (size_t)ch_per_wg_bytes<BITS, UPC, G32, TILES>();
    if (block_bytes < 192 * 1024) per_wg = 1;
    const dim3 grid((n_cblocks + per_wg - 1) / per_wg, max_groups);
    up_gemv_mfma_kernel<BITS, UPC, G32, NTPAD, TILES><<<grid, dim3(kMfmaThreads), lds, stream>>>(table, groups, n_groups, x,
                                                                                                 slots, v, task_tau,
                                                                                                 mask_words, f);
    return hipGetLastError();
}

template <int BITS, int UPC, bool G32>
static hipError_t launch_mfma_chunk(int chunk, int max_groups, hipStream_t stream, const DevExpert* table,
                                    const TokenGroup* groups, const int32_t* n_groups, const h16* x, int slots, float* v,
                                    const float* task_tau, uint32_t* mask_words, int f) {
    if (chunk <= 8) return launch_mfma_inst<BITS, UPC, G32, 8>(max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f);
    return launch_mfma_inst<BITS, UPC, G32, 16>(max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f);
}

template <int BITS, bool G32>
static hipError_t launch_mfma_upc(int upc, int chunk, int max_groups, hipStream_t stream, const DevExpert* table,
                                  const TokenGroup* groups, const int32_t* n_groups, const h16* x, int slots, float* v,
                                  const float* task_tau, uint32_t* mask_words, int f) {
    if (upc == 64) return launch_mfma_chunk<BITS, 64, G32>(chunk, max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f);
    if (upc == 32) return launch_mfma_chunk<BITS, 32, G32>(chunk, max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f);
    return launch_mfma_chunk<BITS, 16, G32>(chunk, max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f);
}

hipError_t launch_up_gemv_grouped(const DevExpert* table, const TokenGroup* groups, const int32_t* n_groups,
                                  int max_groups, int chunk, const h16* x, int slots, float* v, const float* task_tau,
                                  uint32_t* mask_words, int d, int f, int bits, int group, hipStream_t stream) {
    if (!mfma_grouped_shape(d, bits, group) || max_groups <= 0) return hipErrorInvalidValue;
    const int upc = d / 64;
    const bool g32 = group == 32;
    if (bits == 2) return launch_mfma_upc<2, false>(upc, chunk, max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f);
    if (bits == 3)
        return g32 ? launch_mfma_upc<3, true>(upc, chunk, max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f)
                   : launch_mfma_upc<3, false>(upc, chunk, max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f);
    return g32 ? launch_mfma_upc<4, true>(upc, chunk, max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f)
               : launch_mfma_upc<4, false>(upc, chunk, max_groups, stream, table, groups, n_groups, x, slots, v, task_tau, mask_words, f);
}

}  // namespace floe
