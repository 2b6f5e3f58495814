// Internal launcher prototypes (host side).  Launchers validate nothing: shapes are checked once in
// api.hip against the limits each kernel states, before anything is enqueued.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "floe_dev.h"
#include "route.h"
#include "xprep.h"

namespace floe {

// Compute units of the current device (read once per device from its properties; 256 on an MI355X, which is also
// what the host-side size queries assume when no device is usable).
int num_cus();

// true when the packed-fp16 kernel applies to this shape (otherwise the generic kernel runs)
inline bool packed_fast_shape(int d, int bits, int group) {
    return (bits == 2 || bits == 3 || bits == 4) && group >= 32 && (d == 1024 || d == 2048 || d == 4096);
}
__host__ __device__ inline int mask_words_per_task(int f) { return (f + 31) / 32; }

// S0
hipError_t launch_quantize(const h16* w, uint32_t* codes, h16* scale, h16* zero, int d, int f, int bits, int group,
                           hipStream_t stream);

// S2 (+ the comparison of S3): v[task][j] for task in [0, n_tasks); token of a task = task / map.slots.
// task_tau / mask_words: when both are given, bit (j % 32) of mask_words[task][j / 32] = (|v_j| > tau[task]).
// route: when given (INT2, group >= 64, packed shapes, n_experts <= 16 only) the kernel routes in place and
// fills the task table itself; map.task_table and task_tau are then ignored.
hipError_t launch_up_gemv(const TaskMap& map, const h16* x, const RouteArgs* route, float* v, const float* task_tau,
                          uint32_t* mask_words, int d, int f, int bits, int group, int n_tasks, hipStream_t stream);
inline bool route_in_place_ok(int d, int bits, int group, int n_experts, int top_k, int n_shared) {
    return bits == 2 && group >= 64 && packed_fast_shape(d, bits, group) && top_k >= 1 && n_experts <= 16 &&
           top_k + n_shared <= 16;
}

// How the fused kernel gets its routing: 2 = all of S1 inside it (<= 16 experts), 1 = softmax and top-k inside it on
// logits that router_logits computed in front (<= 64 experts: repeated by every workgroup the dot products would cost
// more than that launch), 0 = a router kernel in front writes the task table.
inline int fused_route_mode(int n_experts, int top_k, int n_shared) {
    if (top_k < 1 || top_k + n_shared > 16) return 0;
    return n_experts <= 16 ? 2 : (n_experts <= 64 ? 1 : 0);
}

// (S1 +) S2-S5 of a small decode batch in one kernel (packed shapes, any bit width): every workgroup computes v for
// its own block of channels, selects among them and runs gate/down on what it selected (fused_ffn.h).
// With `route` the workgroup also routes in place (fused_route_mode); otherwise map / task_tau /
// task_scale describe the tasks.  partial[task][blocks][d], wg_count[task][blocks] (selected channels per
// workgroup), v_out (optional) [task][f].
constexpr int fused_producers = 4;                          // producer waves per workgroup (+ 2 consumers each)
constexpr int fused_wgs_per_cu = 1;                         // workgroups per compute unit the block length aims at
// Channel passes per producer wave: a launch argument between these two.  The kernel exists in two sizes, for blocks of
// kFusedMinPasses passes (all of them in flight at once) and for anything up to kFusedMaxPasses (which sizes its queues).
constexpr int kFusedMinPasses = 7, kFusedMaxPasses = 448;
// passes in flight per producer wave: INT2 stages its codes in LDS, as deep as the ring fits the two result slabs it
// borrows (8 d bytes, 1 KiB per pass); INT3 and INT4 hold 4 passes in registers
constexpr int fused_depth(int d, int bits) { return bits == 2 ? (d / 128 < 14 ? d / 128 : 14) : 4; }
constexpr int kFusedMaxRouted = 64;       // routed experts a workgroup can pick among in place (one per lane)
constexpr int kFusedMaxTasks = 256;       // (token, slot) tasks up to which the fused kernel is considered
// Up to how many tasks a layer call takes the fused kernel.  Measured against the batch kernels (grouped up GEMV, union
// gate/down), it wins while experts see few tokens each: config 3 (8 experts) 16 tasks 97 against 132 us, 32 tasks 181
// against 184, 64 tasks 348 against 313; config 5 (66 experts) 64 tasks 38 against 54, 256 tasks 131 against 145.
// Rule: up to 16 tasks always, beyond that up to four tasks per expert.  fused_tasks_tuned() > 0 replaces the rule.
int fused_tasks_tuned();
void set_fused_tasks_tuned(int n);
inline int fused_task_limit(int n_all) {
    const int t = fused_tasks_tuned();
    const int rule = 4 * n_all > 16 ? 4 * n_all : 16;
    const int lim = t > 0 ? t : rule;
    return lim < kFusedMaxTasks ? lim : kFusedMaxTasks;
}
constexpr int kExpertOrderTasks = 16;     // batches of more tasks run their per-task kernels in expert order
constexpr int kFusedMaxWorkgroups = 2048;
struct FusedArgs {
    TaskMap map;
    const h16* x;
    const RouteArgs* route;
    const float* task_tau;
    const float* task_scale;
    float* v_out;
    float* partial;
    int32_t* wg_count;
    int d, f, group, n_tasks, passes;
};
int fused_passes(int d, int f, int bits, int n_tasks, int max_tasks = kExpertOrderTasks);  // 0: not fused
int fused_blocks(int d, int f, int passes);
hipError_t launch_fused(const FusedArgs& a, int bits, hipStream_t stream);

// S2 for decode batches on the matrix cores: tokens routed to the same expert share one pass over its codes.
struct TokenGroup {
    int32_t expert;    // index into the layer's expert table
    int32_t n;         // tasks in this chunk (<= chunk size)
    int32_t task[16];  // ascending task ids (token * slots + slot)
};
inline bool mfma_grouped_shape(int d, int bits, int group) {
    return ((bits == 2 && group == 64) || ((bits == 3 || bits == 4) && (group == 32 || group == 64))) &&
           (d == 1024 || d == 2048 || d == 4096);
}
// tasks per group (token rows of the MFMA tile that are used): 8 while experts see few tokens each, else 16
inline int mfma_chunk(int n_all, int n_tasks) { return n_tasks <= 8 * n_all ? 8 : 16; }
inline int mfma_max_groups(int n_all, int n_tasks) {
    return (n_all < n_tasks ? n_all : n_tasks) + n_tasks / mfma_chunk(n_all, n_tasks) + 1;
}
// Grouping pays once experts see about two tokens each; below that the per-token kernels read the same bytes.  The
// INT3 form is bound by its unpacking and by one round trip per eight units on short channels, not by the bytes: it
// needs three to four tokens per expert before it beats the per-token kernel.  grouped_gemv_mode: 0 = this rule,
// 1 = whenever the shape allows, 2 = never (floe_tuning).
int grouped_gemv_mode();
void set_grouped_gemv_mode(int m);
inline bool mfma_batch_pays(int n_all, int n_tasks, int bits) {
    const int mode = grouped_gemv_mode();
    if (mode == 1) return true;
    if (mode == 2) return false;
    return bits == 3 ? 2 * n_tasks >= 7 * n_all : n_tasks >= 2 * n_all;
}
hipError_t launch_group_tokens(const int32_t* task_expert, int n_tasks, int n_all, int chunk, TokenGroup* groups,
                               int32_t* n_groups, hipStream_t stream, int32_t* order = nullptr);
hipError_t launch_up_gemv_grouped(const DevExpert* table, const TokenGroup* groups, const int32_t* n_groups,
                                  int max_groups, int chunk, const h16* x, int slots, float* v, const float* task_tau,
                                  uint32_t* mask_words, int d, int f, int bits, int group, hipStream_t stream);

// S3 as a kernel of its own: per task threshold tau[task]
hipError_t launch_select(const float* v, int f, int n_tasks, const float* tau, int32_t* idx, int32_t* count,
                         hipStream_t stream);

// S3 (compaction) + S4 + S5.  Index lists come either from mask_words (then idx/count are WRITTEN, both
// may be nullptr) or, with mask_words == nullptr, from idx/count (read).  partial[task][blk][d].
int gd_blocks(int n_tasks, int f);
// staged: nullptr, or the staging buffer [n_tasks][gd_rows][2][d] whose row k of task q holds channel idx[q][k];
// with rows (staged lists only) the k-th channel of task q sits in row rows[q * f + k] of the whole buffer (-1: absent)
hipError_t launch_gate_down(const TaskMap& map, const h16* staged, int gd_rows, const h16* x, const float* v,
                            const uint32_t* mask_words, int32_t* idx, int32_t* count, const float* task_scale,
                            float* partial, int d, int f, int n_tasks, int nblk, hipStream_t stream,
                            const int32_t* rows = nullptr, const int32_t* order = nullptr);

// S4 + S5 for decode batches on the matrix cores, one read of every row that any token of an expert group selected
// (gate_down_union.hip).  The groups are those of launch_group_tokens; mask_words / v come from the GEMV kernels.
struct UnionPlan {
    int nblk_gate, nblk_down;  // channel blocks of the gate kernel; the down kernel takes nblk_gate / nblk_down of them each
    int cap;                   // rows a gate block can hold (a multiple of 16)
    int nt;                    // token rows kept in LDS: 8 or 16 (the group chunk)
    int max_groups;
    bool matrix_cores, fused;  // which kernels run (union_mode)
};
constexpr int kStageWorkgroupsDefault = 32;  // 128 waves x 4 KiB in flight: the link is full, a GEMV beside it keeps most of its speed
int stage_workgroups();
void set_stage_workgroups(int n);  // 0 = default
int union_mode();
int union_kernels_for(int n_all, int n_tasks);  // 1 matrix cores, 2 LDS ring, 3 one-token kernels in expert order
void set_union_mode(int m);
struct UnionArgs {
    const DevExpert* table;
    const TokenGroup* groups;
    const int32_t* n_groups;
    const h16* x;
    const float* v;               // [n_tasks][f]
    const uint32_t* mask_words;   // [n_tasks][words]
    const float* task_scale;      // [n_tasks] or nullptr
    int32_t* count;               // [n_tasks][nblk_gate] selected channels per (task, gate block), or nullptr
    float* partial;               // [n_tasks][nblk_down][d]
    int32_t* urow;                // [max_groups][nblk_gate][cap] union rows, ascending
    int32_t* ucount;              // [max_groups][nblk_gate]
    uint4* hbuf;                  // [max_groups][nblk_gate][cap / 16][64] h fragments (hi, lo) in lane order
    int32_t slots, f, nt, cap, nblk_gate, nblk_down;
};
UnionPlan union_plan(int d, int f, int n_tasks, int n_all, int chunk);
bool union_shape_ok(int d, int f, const UnionPlan& p);
hipError_t launch_gate_down_union(const UnionArgs& a, const UnionPlan& p, int d, hipStream_t stream);

// The other sparsification candidates of Sec. 3.2.1 (variants.hip): act = a_gate (which = 1) or a_down (which = 2) and
// h = a_gate * a_up for every channel; then the down rows of the kept channels only.
hipError_t launch_gate_dense(const h16* gd, const h16* x, const float* v, int which, int d, int f, int T, float* act,
                             float* hval, hipStream_t stream);
hipError_t launch_down_rows(const h16* gd, const float* hval, const int32_t* idx, const int32_t* count,
                            const float* out_scale, int d, int f, int T, int nblk, float* partial, hipStream_t stream);

// S6 (and the "+=" of the one-expert entry points): reduce partial over blocks and slots.
//   y_acc != nullptr: y_acc[t][i] += sum;   y_half != nullptr: y_half[t][i] = fp16(sum)
hipError_t launch_combine(const float* partial, int d, int T, int slots, int nblk, float* y_acc, h16* y_half,
                          hipStream_t stream);

// S1: router + per-task table (resolved expert pointers, weight, tau)
struct RouterArgs {
    const h16* router_cm;
    const h16* x;
    const float* tau;
    int32_t tau_stride_t;
    int32_t n_experts, top_k, n_shared, renormalize, d;
    const DevExpert* table;   // all experts of the layer
    DevExpert* task_table;    // [n_tasks] out
    int32_t* task_expert;     // [n_tasks] out
    float* task_weight;       // [n_tasks] out
    float* task_tau;          // [n_tasks] out
    float* logits;            // [T][n_experts] scratch of the two-launch form; nullptr = one launch always
};
// the router matrix of a token is worth spreading over several workgroups from this size on (two launches then)
inline bool router_split_pays(int n_experts, int d, int T) {
    return (size_t)n_experts * d * 2 >= (size_t)128 * 1024 && n_experts >= 32 && T <= 4096;
}
hipError_t launch_router(const RouterArgs& a, int T, hipStream_t stream);
hipError_t launch_router_logits(const RouterArgs& a, int T, hipStream_t stream);  // x . W_r only, into a.logits

// stats: (expert, count, weight) per task
struct SlotStat {
    int32_t expert;
    int32_t count;
    float weight;
    int32_t staged;
};
// count_parts != 0: the count of task q is the sum of count[q * count_parts .. + count_parts)
// staged (optional): rows of task q that were copied host -> HBM for this call; capacity > 0 clamps it (a list
// longer than the staging slab is truncated)
hipError_t launch_stats(const int32_t* task_expert, const int32_t* count, int count_parts, const float* task_weight,
                        SlotStat* stats, int n_tasks, hipStream_t stream, const int32_t* staged = nullptr, int capacity = 0);

// S7
hipError_t launch_stage(const h16* host_gd_dev, int d, int f, const int32_t* idx, const int32_t* count,
                        int capacity_rows, h16* dst, int32_t* overflow, hipStream_t stream);
// all tasks of a layer at once: source matrix of task q = task_table[q].gd (device view of pinned host memory),
// list idx[q][0..count[q]), destination dst[q][capacity_rows][2][d], overflow[q]
// dst_rows != nullptr: chunk k of task q goes to row dst_rows[q * f + k] of the whole buffer (capacity_rows and
// overflow are then not used: the rows were checked when they were assigned)
hipError_t launch_stage_tasks(const DevExpert* task_table, int d, int f, const int32_t* idx, const int32_t* count,
                              int capacity_rows, h16* dst, int32_t* overflow, int n_tasks, hipStream_t stream,
                              const int32_t* dst_rows = nullptr);

// Prefetch bookkeeping (reuse of the hidden state before layer i for layer i + 1, Sec. 3.3):
// after a predicted list has been staged: row_of[q][j] = k for j = idx[q][k], k < min(count[q], capacity), else -1;
// pred_expert / pred_count receive the predicted expert and the number of rows staged.
hipError_t launch_rowmap(const int32_t* idx, const int32_t* count, const int32_t* task_expert, int f, int capacity_rows,
                         int32_t* row_of, int32_t* pred_expert, int32_t* pred_count, int n_tasks, hipStream_t stream);
// per actual task q: find the predicted task of the same token with the same expert; rows[q][k] = staging row of
// channel idx[q][k] (the predicted one, or a fresh row behind the predicted ones / in the spare slab n_tasks + q);
// misses are listed in miss_idx[q][0..miss_count[q]) with their rows in miss_rows; stat[q] = {matched, predicted, hits, misses}
struct PrefetchStat {
    int32_t expert_predicted, predicted, hits, misses;
};
hipError_t launch_match_rows(const int32_t* idx, const int32_t* count, const int32_t* task_expert, int f, int slots,
                             int capacity_rows, const int32_t* row_of, const int32_t* pred_expert,
                             const int32_t* pred_count, int32_t* rows, int32_t* miss_idx, int32_t* miss_rows,
                             int32_t* miss_count, int32_t* overflow, PrefetchStat* stat, int n_tasks,
                             hipStream_t stream, const int32_t* expert_row_of = nullptr, int miss_first_row = 0);
// Resident-channel cache: with expert_row_of ([n_experts][f], pool row of a resident channel or -1) match_rows looks the
// channels up there instead (rows are rows of the whole pool; the misses of task q go to rows miss_first_row +
// q * capacity_rows + m).  launch_cache_load makes channels resident.
hipError_t launch_cache_load(const DevExpert* table, int expert, int d, int f, const int32_t* idx, const int32_t* count,
                             int first_row, int max_rows, h16* pool, int32_t* row_of, hipStream_t stream);

}  // namespace floe
