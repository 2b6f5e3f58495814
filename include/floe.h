/*
 * floe.h -- C ABI of the MI355X (gfx950) implementation of FloE's compressed sparse expert FFN at decode.
 *
 * The path (paper Sec. 3.2 "Expert Hybrid Compression", Alg. 1 "Efficient Sparse Kernel", Sec. 3.4):
 *   S0  quantize W_up to `bits`-bit group codes (offline)                       Sec. 3.2.2
 *   S1  router: softmax over x.W_r, top-k, optional renormalisation             Sec. 3.3 (first paragraph)
 *   S2  v = x . W_up^Q            (dequant GEMV over all f channels)            Alg. 1 line 2
 *   S3  idx = { j : |v_j| > tau } (ascending), K = |idx|                        Alg. 1 line 3, Eq. 5
 *   S4  h_k = SiLU(x . W_gate[:, idx_k]) * v[idx_k]                             Alg. 1 line 4, Eq. 2
 *   S5  y = sum_k h_k * W_down[idx_k, :]                                        Alg. 1 line 5
 *   S6  out = fp16( sum over selected experts of weight_e * y_e )               Sec. 3.3 (router), Eq. 1
 *   S7  copy the selected [gate column | down row] chunks host -> HBM           Sec. 3.4.2
 *
 * General rules for every entry point
 *  - "dev" pointers are HIP device pointers owned by the CALLER.  The library never allocates, frees
 *    or keeps them.  Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null
 *    stream) and the call returns without synchronising unless stated.
 *  - fp16 values are IEEE binary16 bit patterns (floe_half).  x is a row vector (Eq. 1).
 *  - All matrices are channel-major: row j holds the d numbers of intermediate channel j
 *    (column j of W_up / W_gate, row j of W_down, i.e. W_down is stored transposed as Sec. 3.4.1 asks).
 *    Gate and down are co-located per channel, gd[rows][2][d] (compact layout of Sec. 3.4.2).
 *  - Quantized up projection: codes uint32 [f][d*bits/32], a little-endian bit stream per channel
 *    (code i at bits [bits*i, bits*i+bits)); scale, zero fp16 [f][d/group]; groups run along d.
 *    w_hat = (code - zero) * scale.
 *  - Supported shapes: bits in {1,2,3,4,8} (the widths of the sensitivity study in Sec. 3.2.2; 2, 3 and 4 have
 *    tuned kernels, 1 and 8 run the generic ones); group a power of two in [32, 256]; d % 512 == 0, d <= 8192,
 *    d % group == 0; 1 <= f <= 2^20; 0 <= T <= 4096.  Anything else returns an error code and
 *    enqueues nothing.
 *  - Return value: FLOE_OK (0) or a negative floe_status.  No exceptions, no errno.
 *  - Nothing falls back to the host: if no HIP device is usable every call returns FLOE_EHIP.
 */
#ifndef FLOE_H
#define FLOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t floe_half;

typedef enum {
    FLOE_OK = 0,
    FLOE_EINVAL = -1,       /* NULL pointer, negative size, misaligned buffer */
    FLOE_ESHAPE = -2,       /* d % group != 0, (group*bits) % 32 != 0, d % 512 != 0 ... */
    FLOE_EUNSUPPORTED = -3, /* bits not in {1,2,3,4,8}, group not in {32,64,128,256}, d > 8192 ... */
    FLOE_EWORKSPACE = -4,   /* workspace_bytes smaller than the matching *_workspace_bytes() */
    FLOE_EHIP = -5          /* a HIP runtime call failed (see floe_last_hip_error) */
} floe_status;

typedef struct {
    int32_t d;     /* hidden size (reduction length of up / gate, output length of down) */
    int32_t f;     /* intermediate size = number of channels */
    int32_t bits;  /* code width of the quantized up projection */
    int32_t group; /* quantization group length along d */
} floe_shape;

const char* floe_status_string(int status);
/* hipError_t of the most recent failing HIP call made by this library on the calling thread (0 if none). */
int floe_last_hip_error(void);
/* ABI version, bumped when a struct layout changes. */
int floe_abi_version(void);

/*
 * Measurement hook (no part of the method).  After floe_profile_kernel(id, start, stop) every launch of
 * kernel `id` made from the calling thread records hipEvent_t `start` before and `stop` after it on the
 * launch stream, so a harness can read that kernel's duration with hipEventElapsedTime (this mirrors the
 * per-kernel latency protocol of Sec. 4.1 / Table 1).  id 0 disarms.  The events stay owned by the caller.
 */
typedef enum {
    FLOE_KERNEL_NONE = 0,
    FLOE_KERNEL_QUANTIZE = 1,
    FLOE_KERNEL_ROUTER = 2,
    FLOE_KERNEL_UP_GEMV = 3,
    FLOE_KERNEL_SELECT = 4,
    FLOE_KERNEL_GATE_DOWN = 5,
    FLOE_KERNEL_COMBINE = 6,
    FLOE_KERNEL_STAGE = 7,
    FLOE_KERNEL_FUSED_FFN = 8 /* (router +) up GEMV + selection + gate/down of small batches, one kernel */
} floe_kernel_id;
int floe_profile_kernel(int kernel_id, void* start_event, void* stop_event);

/*
 * Tuning switch (no part of the method; every setting gives results within the same parity bars).
 *   FLOE_TUNE_UNION_KERNELS  how Alg. 1 steps 4-5 run for decode batches (those beyond FLOE_TUNE_FUSED_TASKS), where
 *                            the tokens of an expert select overlapping rows:
 *                            0 = chosen per call (default): 1 once the experts see about a dozen tokens each, else 3;
 *                            1 = per expert group, the union of the selected rows read once, gate and down
 *                                projections on the matrix cores (dense token x row tiles);
 *                            2 = per expert group, the union of the selected rows read once into a ring in LDS, one
 *                                wave per token;
 *                            3 = one workgroup set per (token, slot), launched in expert order on XCD-aligned channel
 *                                blocks, so that a row several tokens selected is fetched from HBM once and served to
 *                                the others by the L2.
 *   FLOE_TUNE_STAGE_WORKGROUPS  workgroups (of four waves, four 16-byte reads in flight per lane) of the kernels that
 *                            copy selected chunks out of pinned host memory; 0 = the library's default, at most 4096.
 *                            More workgroups than the link needs keep more host reads in flight, and these delay the
 *                            HBM reads of kernels that run beside the copy.
 *   FLOE_TUNE_GROUPED_GEMV   decode batches (T >= 2; INT2 g64, INT3 / INT4 g32 or g64; d 1024, 2048 or 4096): whether the
 *                            tokens routed to one expert share one pass over its codes on the matrix cores:
 *                            0 = where the one-kernel path (FLOE_TUNE_FUSED_TASKS) does not apply and measurement says
 *                                it pays (about two tokens per expert; three to four for INT3),
 *                            1 = whenever the shape allows, 2 = never (one pass per (token, slot)).
 *   FLOE_TUNE_FUSED_TASKS    up to how many (token, slot) pairs a layer call runs Alg. 1 in one kernel (every workgroup
 *                            takes a block of channels of one pair through all steps) instead of the batch kernels:
 *                            0 = the library's rule (16, or four per expert if that is more), else the limit itself
 *                            (at most 256).
 * Process-wide.  Workspace sizes depend on FLOE_TUNE_UNION_KERNELS, FLOE_TUNE_GROUPED_GEMV and FLOE_TUNE_FUSED_TASKS: do not change them
 * between a *_workspace_bytes query and the decode call that uses the workspace.  Unknown key or value: FLOE_EINVAL.
 */
typedef enum {
    FLOE_TUNE_UNION_KERNELS = 1,
    FLOE_TUNE_STAGE_WORKGROUPS = 2,
    FLOE_TUNE_GROUPED_GEMV = 3,
    FLOE_TUNE_FUSED_TASKS = 4
} floe_tuning_key;
int floe_tuning(int key, int value);

/* ------------------------------------------------------------------------------------------------
 * S0 -- Sec. 3.2.2.  Asymmetric uniform group quantizer, bit-exact with this definition in IEEE
 * binary32 (one rounding per operation, no fused multiply-add), qmax = 2^bits - 1:
 *   mn, mx = min / max of the group;  scale = fp16_rne((mx - mn) / qmax);  S = (float)scale
 *   zero = fp16_rne(clamp(-mn / S, +-65504));  Z = (float)zero
 *   code = clamp(rint(w / S + Z), 0, qmax)            (rint = ties to even)
 * Degenerate group (mx == mn, or S below 2^-14): scale = 1, zero = fp16_rne(-mn), codes 0.
 * w_up_cm dev [f][d] fp16 in; codes dev [f][d*bits/32], scale dev [f][d/group], zero dev [f][d/group] out.
 */
int floe_quantize_expert(const floe_shape* s, const floe_half* w_up_cm, uint32_t* codes, floe_half* scale,
                         floe_half* zero, void* stream);

/* ------------------------------------------------------------------------------------------------
 * S2 -- Alg. 1 line 2 on the quantized matrix, for T tokens: v[t][j] = sum_i x[t][i] * w_hat[j][i],
 * fp32 accumulation.  x dev [T][d] fp16, v dev [T][f] fp32 (written).
 */
int floe_up_gemv(const floe_shape* s, const uint32_t* codes, const floe_half* scale, const floe_half* zero,
                 const floe_half* x, int T, float* v, void* stream);

/* S3 -- Alg. 1 line 3 for T tokens: idx[t][0..count[t]) = ascending { j : |v[t][j]| > tau[t] }.
 * v dev [T][f]; tau dev [T]; idx dev [T][f] (capacity f per token; entries past count[t] are left
 * untouched); count dev [T].  The comparison is done in binary32 and is strict.
 */
int floe_select_channels(const float* v, int f, int T, const float* tau, int32_t* idx, int32_t* count,
                         void* stream);

/* One compressed expert (plain pointers, no ownership). */
typedef struct {
    floe_shape s;
    const uint32_t* up_codes;  /* dev */
    const floe_half* up_scale; /* dev */
    const floe_half* up_zero;  /* dev */
    const floe_half* gd;       /* dev, compact layout [gd_rows][2][d]: gate column then down row */
    int32_t gd_is_staged;      /* 0: gd_rows == f and row j is channel j;
                                  1: row k holds channel idx[k] (filled by floe_stage_channels) */
    int32_t gd_rows;           /* rows actually present in gd (capacity when staged) */
} floe_expert;

/* Bytes of scratch floe_gate_down_sparse / floe_expert_ffn_sparse need for T tokens of this shape. */
size_t floe_expert_workspace_bytes(const floe_shape* s, int T);

/*
 * S4 + S5 -- Alg. 1 lines 4-5 for T tokens on index lists that already exist:
 *   y_acc[t][:] += out_scale[t] * sum_{k < count[t]} SiLU(x[t] . gate(idx[t][k])) * v[t][idx[t][k]] * down(idx[t][k])
 * v dev [T][f]; idx dev [T][f]; count dev [T]; out_scale dev [T] or NULL (= 1); y_acc dev [T][d] fp32,
 * read-modify-written (the caller zeroes it; this is how the top-k combine of S6 is folded in).
 * With a staged gd, row k of token t's list is read from gd row k, so T must be 1 and count[0] must
 * not exceed gd_rows (rows beyond gd_rows are ignored).
 * workspace: dev, 256-byte aligned, at least floe_expert_workspace_bytes(); contents are scratch.
 */
int floe_gate_down_sparse(const floe_expert* e, const floe_half* x, int T, const float* v, const int32_t* idx,
                          const int32_t* count, const float* out_scale, float* y_acc, void* workspace,
                          size_t workspace_bytes, void* stream);

/*
 * S2..S5 -- the whole of Alg. 1 for one expert and T independent tokens (each token has its own
 * threshold tau[t], its own mask and its own result):
 *   v = x . W_up^Q;  idx, count from |v| > tau;  y_acc += out_scale * (sparse gate/down product).
 * idx dev [T][f] and count dev [T] are outputs (the staging call and the parity checks consume them); pass both
 * as NULL when the list itself is not wanted (the result y_acc is the same; small batches then skip building it).
 * The intermediate v lives in the workspace.  e->gd must be the full (unstaged) matrix.
 */
int floe_expert_ffn_sparse(const floe_expert* e, const floe_half* x, int T, const float* tau,
                           const float* out_scale, float* y_acc, int32_t* idx, int32_t* count, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * The three candidates for sparsification that Sec. 3.2.1 compares (Eq. 3-5): the sparsity function S_t applied to
 *   FLOE_SPARSIFY_UP    a_up = x . W_up^Q            (what FloE uses: identical to floe_expert_ffn_sparse),
 *   FLOE_SPARSIFY_GATE  a_gate = SiLU(x . W_gate),
 *   FLOE_SPARSIFY_DOWN  a_down = a_gate * a_up,
 * inside the expert forward of Eq. 1: y_acc[t] += out_scale[t] * sum over kept channels of a_gate_j a_up_j W_down[j,:],
 * kept = { j : |a_j| > tau[t] } (strict, binary32), written to idx / count as in floe_expert_ffn_sparse (both required
 * for the last two).  With a_gate or a_down the whole gate projection is read before any channel can be dropped and
 * only down rows are saved: these two exist for the comparison of Sec. 3.2.1, not for speed.
 * workspace: floe_expert_sparsified_workspace_bytes().
 */
typedef enum { FLOE_SPARSIFY_UP = 0, FLOE_SPARSIFY_GATE = 1, FLOE_SPARSIFY_DOWN = 2 } floe_sparsify;
size_t floe_expert_sparsified_workspace_bytes(const floe_shape* s, int T);
int floe_expert_ffn_sparsified(const floe_expert* e, int which, const floe_half* x, int T, const float* tau,
                               const float* out_scale, float* y_acc, int32_t* idx, int32_t* count, void* workspace,
                               size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * One MoE layer (S1..S6).  Routed experts come first in `experts`, the n_shared always-on experts
 * (weight 1) follow.  All experts of a layer share one floe_shape.
 */
typedef struct {
    int32_t n_experts, top_k, n_shared, renormalize;
    floe_shape s;
    const floe_half* router_cm; /* dev [n_experts][d] (may be NULL when top_k == 0) */
    const floe_expert* experts; /* HOST array of n_experts + n_shared entries (read by floe_layer_build_table) */
    const float* tau;           /* dev; threshold of (token t, expert e) at tau[t * tau_stride_t + e] */
    int32_t tau_stride_t;       /* n_experts + n_shared for per-token thresholds, 0 to broadcast the
                                   per-expert constant t_ij that Alg. 1 takes as input */
    const void* dev_table;      /* dev, written by floe_layer_build_table: the experts' pointers in HBM */
    int32_t gd_on_host;         /* 0: every expert's gd is in HBM.  1: every expert's gd is PINNED HOST memory
                                   (the offloaded setting of Sec. 3.1 / 3.4.2); only
                                   floe_moe_layer_decode_offloaded accepts such a layer */
} floe_layer;

/* Per (token, slot) record written by floe_moe_layer_decode when `stats` is not NULL;
 * slots 0..top_k-1 are the routed experts by descending probability, then the shared ones. */
typedef struct {
    int32_t expert; /* expert id */
    int32_t count;  /* K: number of selected channels */
    float weight;   /* combine weight */
    int32_t staged; /* rows copied host -> HBM for this (token, slot) by this call (0 for a resident layer).  With chunks
                       of 4*d bytes: bytes touched = count * 4 * d, bytes staged = staged * 4 * d */
} floe_slot_stat;

size_t floe_layer_table_bytes(const floe_layer* L);
/* Copies the experts' device pointers into dev_table (dev, 256-byte aligned, floe_layer_table_bytes()).
 * Every expert's up_codes, up_scale, up_zero and gd must be 16-byte aligned (FLOE_EINVAL otherwise).
 * Synchronises `stream` before returning; L->experts is not read by any later call and may be freed. One-time set-up. */
int floe_layer_build_table(const floe_layer* L, void* dev_table, size_t bytes, void* stream);

size_t floe_layer_workspace_bytes(const floe_layer* L, int T);
/*
 * x dev [T][d] fp16 -> y dev [T][d] fp16.  Router: logits = x . W_r, softmax, top_k (ties to the lower
 * expert id), weights p_e / sum_selected p if renormalize else p_e.  For every (token, selected expert):
 * Alg. 1 with threshold tau[t*tau_stride_t + e]; y[t] = fp16_rne(sum_e weight_e * y_e) accumulated in fp32.
 * stats: dev [T][top_k + n_shared] floe_slot_stat or NULL.  L->dev_table must have been built.
 */
int floe_moe_layer_decode(const floe_layer* L, const floe_half* x, int T, floe_half* y, floe_slot_stat* stats,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same layer decode for callers that cannot allocate device memory or have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Inputs, outputs, results and
 * error codes are those of floe_moe_layer_decode; the workspace is a scratch array of FLOE_STATIC_SCRATCH_BYTES
 * that is part of the library's device image (each GPU the library runs on holds one copy until the process ends).
 * The call allocates and frees nothing.  Limit: floe_layer_workspace_bytes(L, T) must not exceed
 * FLOE_STATIC_SCRATCH_BYTES (ask that function: a Mixtral-shaped layer, d=4096 f=14336 top-2, needs 4.2 MiB per
 * token at T <= 3 and fits again, with other kernels, from T = 9 to about T = 48), otherwise FLOE_EWORKSPACE is
 * returned and nothing is enqueued.  All calls on one GPU share the array: calls that overlap
 * on one GPU (two streams, two threads) race; calls on one stream are ordered and safe.  No kernel relies on what
 * an earlier call left in the array.
 */
#define FLOE_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
int floe_moe_layer_decode_static(const floe_layer* L, const floe_half* x, int T, floe_half* y, floe_slot_stat* stats,
                                 void* stream);

/* ------------------------------------------------------------------------------------------------
 * One MoE layer in the offloaded setting (Sec. 3.1, Fig. 1(c); Sec. 3.4.2): the quantized up projections
 * and the router are resident in HBM, the gate/down matrices stay in pinned host memory and only the
 * selected channels of the routed experts cross the bus.  Sequence:
 *   on `stream`:      router, up GEMV, selection (index lists)           -> ev_lists_ready
 *   on side_stream:   wait ev_lists_ready; copy the selected chunks of every (token, slot) into its slab of
 *                     `staging` (S7)                                     -> ev_staged
 *   on `stream`:      wait ev_staged; gathered gate/down on the staged rows, combine.
 * staging: dev [T * (top_k + n_shared)][capacity_rows][2][d]; a list longer than capacity_rows is truncated
 * and overflow[task] (dev, optional) is set to 1.  The two events are hipEvent_t owned by the caller.
 * L->gd_on_host must be 1 and L->dev_table built by floe_layer_build_table.
 */
typedef struct {
    floe_half* staging;
    int32_t capacity_rows;
    int32_t* overflow;
    void* side_stream;
    void* ev_lists_ready;
    void* ev_staged;
} floe_offload;

int floe_moe_layer_decode_offloaded(const floe_layer* L, const floe_offload* o, const floe_half* x, int T, floe_half* y,
                                    floe_slot_stat* stats, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Prefetching the next layer (intra-expert reuse, Sec. 3.3 and Fig. 1(c)): hidden states of neighbouring layers are
 * alike, so the router and the up projection of layer i + 1 applied to the input of layer i predict which experts
 * layer i + 1 will route to and which of their channels will pass the threshold.
 *
 * floe_moe_layer_prefetch: on p->prefetch_stream, after everything enqueued on `stream` so far (x_cur is valid there):
 *   router, up GEMV and selection of layer L on x_cur; the selected chunks of every predicted (token, slot) are copied
 *   from pinned host memory into slab q = token * slots + slot of p->staging (at most capacity_rows each);
 *   p->pred_expert[q], p->pred_count[q] and p->row_of[q][j] (staging row of channel j, -1 = not staged) describe them;
 *   p->ev_prefetched is recorded when all of that is in place.  workspace: floe_layer_workspace_bytes(L, T), NOT the
 *   one a decode call may be using at the same time.
 * floe_moe_layer_decode_prefetched: the layer's real input x on `stream`: router, up GEMV, selection; then, per
 *   (token, slot): the predicted slab of the same token that holds the same expert is reused - its hits stay where they
 *   are, the misses get fresh rows behind them - and an expert that was not predicted takes a spare slab
 *   (p->staging has 2 * T * slots slabs).  Only the misses cross the bus (m->miss_stream); gate/down and combine follow
 *   on `stream`.  Results are identical to floe_moe_layer_decode_offloaded unless a slab overflows
 *   (m->overflow[q] = 1: channels without a row are left out).  prefetch_stats: dev [T * slots] or NULL.
 * Buffers: staging dev [2 * T * slots][capacity_rows][2][d]; pred_expert, pred_count dev [T * slots];
 * row_of dev [T * slots][f]; events are hipEvent_t owned by the caller; two floe_prefetch objects alternate between
 * neighbouring layers.
 */
typedef struct {
    floe_half* staging;
    int32_t capacity_rows;
    int32_t* pred_expert;
    int32_t* pred_count;
    int32_t* row_of;
    void* prefetch_stream;
    void* ev_inputs_ready;
    void* ev_prefetched;
} floe_prefetch;

typedef struct {
    void* miss_stream;
    void* ev_lists_ready;
    void* ev_staged;
    int32_t* overflow; /* dev [T * slots] or NULL */
} floe_miss_path;

typedef struct {
    int32_t expert_predicted; /* 1: a predicted slab of the token held this expert */
    int32_t predicted;        /* channels that were staged ahead for it */
    int32_t hits;             /* selected channels found among them */
    int32_t misses;           /* selected channels that had to be copied now */
} floe_prefetch_stat;

int floe_moe_layer_prefetch(const floe_layer* L, const floe_prefetch* p, const floe_half* x_cur, int T, void* workspace,
                            size_t workspace_bytes, void* stream);
int floe_moe_layer_decode_prefetched(const floe_layer* L, const floe_prefetch* p, const floe_miss_path* m,
                                     const floe_half* x, int T, floe_half* y, floe_slot_stat* stats,
                                     floe_prefetch_stat* prefetch_stats, void* workspace, size_t workspace_bytes,
                                     void* stream);

/* ------------------------------------------------------------------------------------------------
 * Resident channels under a memory budget ("with additional VRAM, we cache more ...", Sec. 4.1): some [gate | down]
 * chunks of an offloaded layer are kept in HBM, and a decode call copies only the selected channels that are not.
 * Which channels are kept is the caller's policy; the paper gives none.
 *   pool          dev [resident_rows + T * slots * capacity_rows][2][d]: the resident chunks first, then one slab of
 *                 capacity_rows rows per (token, slot) for the chunks that have to be copied
 *   row_of        dev [n_experts + n_shared][f]: pool row of channel j of expert e, or -1 (the caller fills it with -1
 *                 once; floe_channel_cache_load enters the rows it writes)
 * floe_channel_cache_load: channels idx[0 .. min(count[0], max_rows)) (dev) of `expert` are copied from its pinned host
 *   matrix to pool rows first_row, first_row + 1, ... (byte copies) and entered in row_of; first_row + max_rows must not
 *   exceed resident_rows.  A channel loaded twice keeps its latest row.
 * floe_moe_layer_decode_cached: as floe_moe_layer_decode_offloaded, but a selected channel with a resident row is read
 *   there and only the others cross the bus (m->miss_stream) into the task's slab; more misses than capacity_rows:
 *   m->overflow[q] = 1 and the channels without a row are left out.  cache_stats (dev [T * slots] or NULL): hits, misses.
 *   Results are identical to floe_moe_layer_decode_offloaded (same kernels, same order of summation).
 */
typedef struct {
    floe_half* pool;
    int32_t* row_of;
    int32_t resident_rows;
    int32_t capacity_rows;
} floe_channel_cache;

int floe_channel_cache_load(const floe_layer* L, const floe_channel_cache* c, int expert, const int32_t* idx,
                            const int32_t* count, int first_row, int max_rows, void* stream);
int floe_moe_layer_decode_cached(const floe_layer* L, const floe_channel_cache* c, const floe_miss_path* m,
                                 const floe_half* x, int T, floe_half* y, floe_slot_stat* stats,
                                 floe_prefetch_stat* cache_stats, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * S7 -- Sec. 3.4.2 (compact asynchronous transfer), done the MI355X way: a copy kernel on a side
 * stream reads the selected 4*d-byte [gate | down] chunks straight out of pinned, device-mapped host
 * memory, so the device-resident index list never travels to the host.
 *   for k < min(count[0], capacity_rows):  hbm_dst[k][:][:] = host_gd[idx[k]][:][:]
 * host_gd: pinned host memory [f][2][d] (hipHostMalloc / torch pin_memory); idx, count: dev.
 * List entries outside [0, f) are skipped (their destination rows are left untouched).
 * overflow: dev int32 or NULL; set to 1 when count[0] > capacity_rows (the extra rows are skipped), else 0.
 * done: a hipEvent_t (as void*) recorded on side_stream after the copy, or NULL.
 */
int floe_stage_channels(const floe_half* host_gd, int d, int f, const int32_t* idx, const int32_t* count,
                        int capacity_rows, floe_half* hbm_dst, int32_t* overflow, void* side_stream, void* done);

#ifdef __cplusplus
}
#endif
#endif /* FLOE_H */
