// C ABI of the library (declared in include/floe.h): argument checks, workspace carving, launches.
// Nothing here computes on the host, and there is no host fallback: without a usable HIP device the
// launches fail and the error is returned.
#include "../../include/floe.h"

#include <hip/hip_runtime.h>

#include <vector>

#include "launch.h"

using namespace floe;

static_assert(sizeof(floe_slot_stat) == sizeof(SlotStat), "stat record layout");
static_assert(sizeof(DevExpert) == 32, "expert table entry");

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return FLOE_EHIP;
}

#define FLOE_HIP(call)                             \
    do {                                           \
        hipError_t e__ = (call);                   \
        if (e__ != hipSuccess) return hip_fail(e__); \
    } while (0)

// Optional measurement hook: when armed for kernel `id`, the next launches of that kernel are bracketed
// by the two events on the launch stream (see floe_profile_kernel in floe.h).
struct ProfileHook {
    int id = 0;
    hipEvent_t start = nullptr, stop = nullptr;
};
thread_local ProfileHook g_hook;

struct Bracket {
    bool on;
    hipStream_t st;
    Bracket(int id, hipStream_t s) : on(g_hook.id == id && g_hook.start && g_hook.stop), st(s) {
        if (on) (void)hipEventRecord(g_hook.start, st);
    }
    ~Bracket() {
        if (on) (void)hipEventRecord(g_hook.stop, st);
    }
};

#define FLOE_LAUNCH(id, stream, call) \
    do {                              \
        Bracket br__((id), (stream)); \
        FLOE_HIP(call);               \
    } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_shape(const floe_shape* s) {
    if (!s) return FLOE_EINVAL;
    if (s->d <= 0 || s->f <= 0 || s->group <= 0) return FLOE_EINVAL;
    if (s->bits != 1 && s->bits != 2 && s->bits != 3 && s->bits != 4 && s->bits != 8) return FLOE_EUNSUPPORTED;
    if (s->group != 32 && s->group != 64 && s->group != 128 && s->group != 256) return FLOE_EUNSUPPORTED;
    if (s->d % s->group != 0) return FLOE_ESHAPE;
    if ((s->group * s->bits) % 32 != 0) return FLOE_ESHAPE;
    if (s->d % 512 != 0) return FLOE_ESHAPE;
    if (s->d > 8192) return FLOE_EUNSUPPORTED;
    if (s->f > (1 << 20)) return FLOE_EUNSUPPORTED;
    return FLOE_OK;
}

int check_T(int T) {
    if (T < 0) return FLOE_EINVAL;
    if (T > 4096) return FLOE_EUNSUPPORTED;
    return FLOE_OK;
}

TaskMap single_map(const floe_expert* e) {
    TaskMap m;
    m.single.codes = e->up_codes;
    m.single.scale = reinterpret_cast<const h16*>(e->up_scale);
    m.single.zero = reinterpret_cast<const h16*>(e->up_zero);
    m.single.gd = reinterpret_cast<const h16*>(e->gd);
    m.task_table = nullptr;
    m.slots = 1;
    return m;
}

// workspace of the one-expert entry points: [v: T*f floats][mask words][counts][idx when not fused][partial: T*nblk*d floats]
struct ExpertWs {
    size_t v_off, mask_off, count_off, idx_off, partial_off, total;
    int nblk, fused_passes, nblk_fused;
};
ExpertWs expert_ws(const floe_shape* s, int T) {
    ExpertWs w;
    w.nblk = gd_blocks(T, s->f);
    w.fused_passes = packed_fast_shape(s->d, s->bits, s->group) ? fused_passes(s->d, s->f, s->bits, T) : 0;
    w.nblk_fused = w.fused_passes ? fused_blocks(s->d, s->f, w.fused_passes) : 0;
    const int nblk_alloc = w.nblk > w.nblk_fused ? w.nblk : w.nblk_fused;
    size_t o = 0;
    w.v_off = o;       o += align_up((size_t)T * s->f * sizeof(float));
    w.mask_off = o;    o += align_up((size_t)T * mask_words_per_task(s->f) * sizeof(uint32_t));
    w.count_off = o;   o += align_up((size_t)T * (w.nblk_fused > 1 ? w.nblk_fused : 1) * sizeof(int32_t));
    w.idx_off = o;     o += w.fused_passes ? 0 : align_up((size_t)T * s->f * sizeof(int32_t));  // list for callers that pass none
    w.partial_off = o; o += align_up((size_t)T * nblk_alloc * s->d * sizeof(float));
    w.total = o;
    return w;
}

// lists longer than this are compacted by the select kernel instead of inside the gate/down kernel
bool mask_path_ok(int f) { return mask_words_per_task(f) <= 2048; }

// workspace of the layer: per-task table, counts, mask words, v, idx, partial
struct LayerWs {
    size_t table_off, expert_off, weight_off, tau_off, logit_off, count_off, mask_off, groups_off, ngroups_off, order_off, v_off, idx_off,
        rows_off, missidx_off, missrows_off, misscount_off, urow_off, ucount_off, hbuf_off, partial_off, total;
    int n_tasks, nblk, nblk_fused, fused_passes;
    bool batch_mfma;  // tokens of an expert share one pass over its codes (matrix-core up GEMV)
    bool use_union;   // batches: one read of every row an expert group selected (gate_down_union.hip)
    int chunk;        // tasks per token group
    UnionPlan up;
};
LayerWs layer_ws(const floe_layer* L, int T) {
    LayerWs w;
    const int slots = L->top_k + L->n_shared;
    w.n_tasks = T * slots;
    w.nblk = gd_blocks(w.n_tasks, L->s.f);
    const int n_all = L->n_experts + L->n_shared;
    w.fused_passes = packed_fast_shape(L->s.d, L->s.bits, L->s.group)
                         ? fused_passes(L->s.d, L->s.f, L->s.bits, w.n_tasks, fused_task_limit(n_all)) : 0;
    w.nblk_fused = w.fused_passes ? fused_blocks(L->s.d, L->s.f, w.fused_passes) : 0;
    w.chunk = mfma_chunk(n_all, w.n_tasks);
    w.up = union_plan(L->s.d, L->s.f, w.n_tasks, n_all, w.chunk);
    // the grouped up GEMV: when forced, or where the fused kernel does not apply and grouping pays
    w.batch_mfma = T >= 2 && mfma_grouped_shape(L->s.d, L->s.bits, L->s.group) &&
                   (grouped_gemv_mode() == 1 || (!w.fused_passes && mfma_batch_pays(n_all, w.n_tasks, L->s.bits)));
    w.use_union = union_kernels_for(n_all, w.n_tasks) != 3 && !L->gd_on_host && T >= 2 && (!w.fused_passes || w.batch_mfma) &&
                  mask_path_ok(L->s.f) && union_shape_ok(L->s.d, L->s.f, w.up);
    int nblk_alloc = w.nblk > w.nblk_fused ? w.nblk : w.nblk_fused;
    if (w.use_union && w.up.nblk_down > nblk_alloc) nblk_alloc = w.up.nblk_down;
    int count_parts = w.nblk_fused > 1 ? w.nblk_fused : 1;
    if (w.use_union && w.up.nblk_gate > count_parts) count_parts = w.up.nblk_gate;
    size_t o = 0;
    w.table_off = o;  o += align_up((size_t)w.n_tasks * sizeof(DevExpert));
    w.expert_off = o; o += align_up((size_t)w.n_tasks * 4);
    w.weight_off = o; o += align_up((size_t)w.n_tasks * 4);
    w.tau_off = o;    o += align_up((size_t)w.n_tasks * 4);
    // router logits in memory: between the two launches of a split router, or in front of a fused kernel that picks in place
    const bool logits_kept = router_split_pays(L->n_experts, L->s.d, T) ||
                             (w.fused_passes && fused_route_mode(L->n_experts, L->top_k, L->n_shared) == 1);
    w.logit_off = o;  o += logits_kept ? align_up((size_t)T * L->n_experts * 4) : 0;
    w.count_off = o;  o += align_up((size_t)w.n_tasks * count_parts * 4);
    w.mask_off = o;   o += align_up((size_t)w.n_tasks * mask_words_per_task(L->s.f) * 4);
    w.groups_off = o; o += align_up((size_t)mfma_max_groups(L->n_experts + L->n_shared, w.n_tasks) * sizeof(TokenGroup));
    w.ngroups_off = o; o += align_up(4);
    w.order_off = o;   o += align_up((size_t)w.n_tasks * 4);
    w.v_off = o;      o += align_up((size_t)w.n_tasks * L->s.f * 4);
    w.idx_off = o;    o += align_up((size_t)w.n_tasks * L->s.f * 4);
    // host-resident gate/down: row map and miss lists of the prefetched decode
    const size_t per_list = L->gd_on_host ? align_up((size_t)w.n_tasks * L->s.f * 4) : 0;
    w.rows_off = o;      o += per_list;
    w.missidx_off = o;   o += per_list;
    w.missrows_off = o;  o += per_list;
    w.misscount_off = o; o += L->gd_on_host ? align_up((size_t)w.n_tasks * 4) : 0;
    const size_t gblocks = w.use_union ? (size_t)w.up.max_groups * w.up.nblk_gate : 0;
    w.urow_off = o;   o += w.use_union ? align_up(gblocks * w.up.cap * 4) : 0;
    w.ucount_off = o; o += w.use_union ? align_up(gblocks * 4) : 0;
    w.hbuf_off = o;   o += w.use_union ? align_up(gblocks * (w.up.cap / 16) * 64 * sizeof(uint4)) : 0;
    w.partial_off = o; o += align_up((size_t)w.n_tasks * nblk_alloc * L->s.d * 4);
    w.total = o;
    return w;
}

int check_layer(const floe_layer* L) {
    if (!L) return FLOE_EINVAL;
    int rc = check_shape(&L->s);
    if (rc) return rc;
    if (L->n_experts < 0 || L->top_k < 0 || L->n_shared < 0) return FLOE_EINVAL;
    if (L->top_k > L->n_experts) return FLOE_EINVAL;
    if (L->top_k + L->n_shared <= 0) return FLOE_EINVAL;
    if (L->n_experts > 1024 || L->top_k + L->n_shared > 64) return FLOE_EUNSUPPORTED;
    if (L->top_k > 0 && !L->router_cm) return FLOE_EINVAL;
    if (!L->tau) return FLOE_EINVAL;
    if (L->tau_stride_t != 0 && L->tau_stride_t != L->n_experts + L->n_shared) return FLOE_EINVAL;
    return FLOE_OK;
}

// arguments of the stand-alone router: it fills the per-task arrays at the head of the workspace
RouterArgs router_args(const floe_layer* L, const LayerWs& w, char* base, const h16* xh) {
    RouterArgs ra;
    ra.router_cm = reinterpret_cast<const h16*>(L->router_cm);
    ra.x = xh;
    ra.tau = L->tau;
    ra.tau_stride_t = L->tau_stride_t;
    ra.n_experts = L->n_experts; ra.top_k = L->top_k; ra.n_shared = L->n_shared; ra.renormalize = L->renormalize;
    ra.d = L->s.d;
    ra.table = static_cast<const DevExpert*>(L->dev_table);
    ra.task_table = reinterpret_cast<DevExpert*>(base + w.table_off);
    ra.task_expert = reinterpret_cast<int32_t*>(base + w.expert_off);
    ra.task_weight = reinterpret_cast<float*>(base + w.weight_off);
    ra.task_tau = reinterpret_cast<float*>(base + w.tau_off);
    ra.logits = w.logit_off != w.count_off ? reinterpret_cast<float*>(base + w.logit_off) : nullptr;
    return ra;
}

// S1-S3 of a layer as separate results in the workspace (offloaded paths need the index lists in memory):
// task table / expert / weight / tau, v, idx, count.
int layer_lists(const floe_layer* L, const LayerWs& w, char* base, const h16* xh, int T, hipStream_t st) {
    DevExpert* task_table = reinterpret_cast<DevExpert*>(base + w.table_off);
    int32_t* task_expert = reinterpret_cast<int32_t*>(base + w.expert_off);
    float* task_weight = reinterpret_cast<float*>(base + w.weight_off);
    float* task_tau = reinterpret_cast<float*>(base + w.tau_off);
    int32_t* count = reinterpret_cast<int32_t*>(base + w.count_off);
    float* v = reinterpret_cast<float*>(base + w.v_off);
    int32_t* idx = reinterpret_cast<int32_t*>(base + w.idx_off);
    TaskMap map{};
    map.task_table = task_table;
    map.slots = L->top_k + L->n_shared;
    if (route_in_place_ok(L->s.d, L->s.bits, L->s.group, L->n_experts, L->top_k, L->n_shared)) {
        RouteArgs ro{};
        ro.router_cm = reinterpret_cast<const h16*>(L->router_cm);
        ro.tau = L->tau;
        ro.tau_stride_t = L->tau_stride_t;
        ro.n_experts = L->n_experts; ro.top_k = L->top_k; ro.n_shared = L->n_shared; ro.renormalize = L->renormalize;
        ro.table = static_cast<const DevExpert*>(L->dev_table);
        ro.task_table = task_table;
        ro.task_expert = task_expert; ro.task_weight = task_weight; ro.task_tau = task_tau;
        FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                    launch_up_gemv(map, xh, &ro, v, nullptr, nullptr, L->s.d, L->s.f, L->s.bits, L->s.group,
                                   w.n_tasks, st));
    } else {
        const RouterArgs ra = router_args(L, w, base, xh);
        FLOE_LAUNCH(FLOE_KERNEL_ROUTER, st, launch_router(ra, T, st));
        FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                    launch_up_gemv(map, xh, nullptr, v, nullptr, nullptr, L->s.d, L->s.f, L->s.bits, L->s.group,
                                   w.n_tasks, st));
    }
    FLOE_LAUNCH(FLOE_KERNEL_SELECT, st, launch_select(v, L->s.f, w.n_tasks, task_tau, idx, count, st));
    return FLOE_OK;
}

}  // namespace

extern "C" {

const char* floe_status_string(int status) {
    switch (status) {
        case FLOE_OK: return "ok";
        case FLOE_EINVAL: return "invalid argument (null pointer, negative size or misaligned buffer)";
        case FLOE_ESHAPE: return "shape violates a divisibility rule (d % group, group*bits % 32, d % 512)";
        case FLOE_EUNSUPPORTED: return "unsupported configuration (bits, group, d, f, T or expert count out of range)";
        case FLOE_EWORKSPACE: return "workspace too small";
        case FLOE_EHIP: return "HIP runtime error (see floe_last_hip_error)";
        default: return "unknown status";
    }
}

int floe_last_hip_error(void) { return g_last_hip_error; }
int floe_abi_version(void) { return 4; }

int floe_profile_kernel(int kernel_id, void* start_event, void* stop_event) {
    if (kernel_id < 0 || kernel_id > FLOE_KERNEL_FUSED_FFN) return FLOE_EINVAL;
    if (kernel_id != 0 && (!start_event || !stop_event)) return FLOE_EINVAL;
    g_hook.id = kernel_id;
    g_hook.start = (hipEvent_t)start_event;
    g_hook.stop = (hipEvent_t)stop_event;
    return FLOE_OK;
}

int floe_tuning(int key, int value) {
    switch (key) {
        case FLOE_TUNE_UNION_KERNELS:
            if (value < 0 || value > 3) return FLOE_EINVAL;
            set_union_mode(value);
            return FLOE_OK;
        case FLOE_TUNE_GROUPED_GEMV:
            if (value < 0 || value > 2) return FLOE_EINVAL;
            set_grouped_gemv_mode(value);
            return FLOE_OK;
        case FLOE_TUNE_FUSED_TASKS:
            if (value < 0 || value > kFusedMaxTasks) return FLOE_EINVAL;
            set_fused_tasks_tuned(value);
            return FLOE_OK;
        case FLOE_TUNE_STAGE_WORKGROUPS:
            if (value < 0 || value > 4096) return FLOE_EINVAL;
            set_stage_workgroups(value);
            return FLOE_OK;
        default: return FLOE_EINVAL;
    }
}

int floe_quantize_expert(const floe_shape* s, const floe_half* w_up_cm, uint32_t* codes, floe_half* scale,
                         floe_half* zero, void* stream) {
    int rc = check_shape(s);
    if (rc) return rc;
    if (!w_up_cm || !codes || !scale || !zero) return FLOE_EINVAL;
    if (!aligned(w_up_cm, 16) || !aligned(codes, 4) || !aligned(scale, 2) || !aligned(zero, 2)) return FLOE_EINVAL;
    FLOE_LAUNCH(FLOE_KERNEL_QUANTIZE, (hipStream_t)stream, launch_quantize(reinterpret_cast<const h16*>(w_up_cm), codes, reinterpret_cast<h16*>(scale),
                             reinterpret_cast<h16*>(zero), s->d, s->f, s->bits, s->group, (hipStream_t)stream));
    return FLOE_OK;
}

int floe_up_gemv(const floe_shape* s, const uint32_t* codes, const floe_half* scale, const floe_half* zero,
                 const floe_half* x, int T, float* v, void* stream) {
    int rc = check_shape(s);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;  // empty batch: pointers of empty arrays may be NULL
    if (!codes || !scale || !zero || !x || !v) return FLOE_EINVAL;
    if (!aligned(codes, 16) || !aligned(x, 16) || !aligned(v, 4)) return FLOE_EINVAL;
    floe_expert e{};
    e.up_codes = codes; e.up_scale = scale; e.up_zero = zero;
    FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, (hipStream_t)stream,
                launch_up_gemv(single_map(&e), reinterpret_cast<const h16*>(x), nullptr, v, nullptr, nullptr, s->d, s->f,
                               s->bits, s->group, T, (hipStream_t)stream));
    return FLOE_OK;
}

int floe_select_channels(const float* v, int f, int T, const float* tau, int32_t* idx, int32_t* count, void* stream) {
    if (f <= 0) return FLOE_EINVAL;
    if (f > (1 << 20)) return FLOE_EUNSUPPORTED;
    int rc = check_T(T);
    if (rc) return rc;
    if (T == 0) return FLOE_OK;
    if (!v || !tau || !idx || !count) return FLOE_EINVAL;
    FLOE_LAUNCH(FLOE_KERNEL_SELECT, (hipStream_t)stream, launch_select(v, f, T, tau, idx, count, (hipStream_t)stream));
    return FLOE_OK;
}

size_t floe_expert_workspace_bytes(const floe_shape* s, int T) {
    if (check_shape(s) != FLOE_OK || T < 0) return 0;
    return expert_ws(s, T).total;
}

int floe_gate_down_sparse(const floe_expert* e, const floe_half* x, int T, const float* v, const int32_t* idx,
                          const int32_t* count, const float* out_scale, float* y_acc, void* workspace,
                          size_t workspace_bytes, void* stream) {
    if (!e) return FLOE_EINVAL;
    int rc = check_shape(&e->s);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;
    if (!e->gd || !x || !v || !idx || !count || !y_acc || !workspace) return FLOE_EINVAL;
    if (!aligned(e->gd, 16) || !aligned(x, 16) || !aligned(y_acc, 16) || !aligned(workspace, kAlign)) return FLOE_EINVAL;
    if (e->gd_is_staged && (T > 1 || e->gd_rows < 0)) return FLOE_EINVAL;
    if (!e->gd_is_staged && e->gd_rows != e->s.f) return FLOE_EINVAL;
    const ExpertWs w = expert_ws(&e->s, T);
    if (workspace_bytes < w.total) return FLOE_EWORKSPACE;
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.partial_off);
    hipStream_t st = (hipStream_t)stream;
    FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st, launch_gate_down(single_map(e), e->gd_is_staged ? reinterpret_cast<const h16*>(e->gd) : nullptr, e->gd_rows,
                              reinterpret_cast<const h16*>(x), v, nullptr,
                              const_cast<int32_t*>(idx), const_cast<int32_t*>(count), out_scale, partial, e->s.d, e->s.f, T, w.nblk, st));
    FLOE_LAUNCH(FLOE_KERNEL_COMBINE, st, launch_combine(partial, e->s.d, T, 1, w.nblk, y_acc, nullptr, st));
    return FLOE_OK;
}

int floe_expert_ffn_sparse(const floe_expert* e, const floe_half* x, int T, const float* tau, const float* out_scale,
                           float* y_acc, int32_t* idx, int32_t* count, void* workspace, size_t workspace_bytes,
                           void* stream) {
    if (!e) return FLOE_EINVAL;
    int rc = check_shape(&e->s);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;
    if (!e->up_codes || !e->up_scale || !e->up_zero || !e->gd || !x || !tau || !y_acc || !workspace) return FLOE_EINVAL;
    if ((idx == nullptr) != (count == nullptr)) return FLOE_EINVAL;  // the list and its length come together
    if (!aligned(e->up_codes, 16) || !aligned(e->gd, 16) || !aligned(x, 16) || !aligned(y_acc, 16) ||
        !aligned(workspace, kAlign))
        return FLOE_EINVAL;
    if (e->gd_is_staged || e->gd_rows != e->s.f) return FLOE_EINVAL;
    const ExpertWs w = expert_ws(&e->s, T);
    if (workspace_bytes < w.total) return FLOE_EWORKSPACE;
    float* v = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.v_off);
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.partial_off);
    hipStream_t st = (hipStream_t)stream;
    const TaskMap map = single_map(e);
    const h16* xh = reinterpret_cast<const h16*>(x);
    uint32_t* mask = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + w.mask_off);
    int nblk = w.nblk;
    if (w.fused_passes) {
        // small batch: GEMV, selection and gate/down in one kernel; the list, when asked for, is cut from v afterwards
        FusedArgs a{};
        a.map = map; a.x = xh; a.route = nullptr; a.task_tau = tau; a.task_scale = out_scale;
        a.v_out = idx ? v : nullptr;
        a.partial = partial;
        a.wg_count = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + w.count_off);
        a.d = e->s.d; a.f = e->s.f; a.group = e->s.group; a.n_tasks = T; a.passes = w.fused_passes;
        FLOE_LAUNCH(FLOE_KERNEL_FUSED_FFN, st, launch_fused(a, e->s.bits, st));
        if (idx) FLOE_LAUNCH(FLOE_KERNEL_SELECT, st, launch_select(v, e->s.f, T, tau, idx, count, st));
        nblk = w.nblk_fused;
    } else {
        // a caller that wants no list still gets one built, in the workspace
        int32_t* idx_ws = idx ? idx : reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + w.idx_off);
        int32_t* count_ws = count ? count : reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + w.count_off);
        if (mask_path_ok(e->s.f)) {
            // the GEMV leaves one mask bit per channel; the gate/down kernel compacts them and writes idx / count
            FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                        launch_up_gemv(map, xh, nullptr, v, tau, mask, e->s.d, e->s.f, e->s.bits, e->s.group, T, st));
            FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                        launch_gate_down(map, nullptr, e->s.f, xh, v, mask, idx_ws, count_ws, out_scale, partial, e->s.d,
                                         e->s.f, T, w.nblk, st));
        } else {
            FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                        launch_up_gemv(map, xh, nullptr, v, nullptr, nullptr, e->s.d, e->s.f, e->s.bits, e->s.group, T, st));
            FLOE_LAUNCH(FLOE_KERNEL_SELECT, st, launch_select(v, e->s.f, T, tau, idx_ws, count_ws, st));
            FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                        launch_gate_down(map, nullptr, e->s.f, xh, v, nullptr, idx_ws, count_ws, out_scale, partial, e->s.d,
                                         e->s.f, T, w.nblk, st));
        }
    }
    FLOE_LAUNCH(FLOE_KERNEL_COMBINE, st, launch_combine(partial, e->s.d, T, 1, nblk, y_acc, nullptr, st));
    return FLOE_OK;
}

// workspace of the sparsification variants: [v][act][h: T*f floats each][partial: T*nblk*d floats]
namespace {
struct VariantWs {
    size_t v_off, act_off, h_off, partial_off, total;
    int nblk;
};
VariantWs variant_ws(const floe_shape* s, int T) {
    VariantWs w;
    w.nblk = gd_blocks(T, s->f);
    size_t o = 0;
    w.v_off = o;       o += align_up((size_t)T * s->f * 4);
    w.act_off = o;     o += align_up((size_t)T * s->f * 4);
    w.h_off = o;       o += align_up((size_t)T * s->f * 4);
    w.partial_off = o; o += align_up((size_t)T * w.nblk * s->d * 4);
    w.total = o;
    return w;
}
}  // namespace

size_t floe_expert_sparsified_workspace_bytes(const floe_shape* s, int T) {
    if (check_shape(s) != FLOE_OK || T < 0) return 0;
    const size_t a = expert_ws(s, T).total, b = variant_ws(s, T).total;
    return a > b ? a : b;
}

int floe_expert_ffn_sparsified(const floe_expert* e, int which, const floe_half* x, int T, const float* tau,
                               const float* out_scale, float* y_acc, int32_t* idx, int32_t* count, void* workspace,
                               size_t workspace_bytes, void* stream) {
    if (which == FLOE_SPARSIFY_UP)
        return floe_expert_ffn_sparse(e, x, T, tau, out_scale, y_acc, idx, count, workspace, workspace_bytes, stream);
    if (which != FLOE_SPARSIFY_GATE && which != FLOE_SPARSIFY_DOWN) return FLOE_EINVAL;
    if (!e) return FLOE_EINVAL;
    int rc = check_shape(&e->s);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;
    if (!e->up_codes || !e->up_scale || !e->up_zero || !e->gd || !x || !tau || !y_acc || !idx || !count || !workspace)
        return FLOE_EINVAL;
    if (!aligned(e->up_codes, 16) || !aligned(e->gd, 16) || !aligned(x, 16) || !aligned(y_acc, 16) ||
        !aligned(workspace, kAlign))
        return FLOE_EINVAL;
    if (e->gd_is_staged || e->gd_rows != e->s.f) return FLOE_EINVAL;
    const VariantWs w = variant_ws(&e->s, T);
    if (workspace_bytes < w.total) return FLOE_EWORKSPACE;
    char* base = static_cast<char*>(workspace);
    float* v = reinterpret_cast<float*>(base + w.v_off);
    float* act = reinterpret_cast<float*>(base + w.act_off);
    float* hval = reinterpret_cast<float*>(base + w.h_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = (hipStream_t)stream;
    const h16* xh = reinterpret_cast<const h16*>(x);
    const h16* gd = reinterpret_cast<const h16*>(e->gd);
    // a_up for every channel (the quantized up projection), a_gate for every channel, the chosen activation against t,
    // then only the down rows of the channels that are kept
    FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                launch_up_gemv(single_map(e), xh, nullptr, v, nullptr, nullptr, e->s.d, e->s.f, e->s.bits, e->s.group, T, st));
    FLOE_HIP(launch_gate_dense(gd, xh, v, which, e->s.d, e->s.f, T, act, hval, st));
    FLOE_LAUNCH(FLOE_KERNEL_SELECT, st, launch_select(act, e->s.f, T, tau, idx, count, st));
    FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                launch_down_rows(gd, hval, idx, count, out_scale, e->s.d, e->s.f, T, w.nblk, partial, st));
    FLOE_LAUNCH(FLOE_KERNEL_COMBINE, st, launch_combine(partial, e->s.d, T, 1, w.nblk, y_acc, nullptr, st));
    return FLOE_OK;
}

size_t floe_layer_table_bytes(const floe_layer* L) {
    if (!L || L->n_experts < 0 || L->n_shared < 0) return 0;
    return align_up((size_t)(L->n_experts + L->n_shared) * sizeof(DevExpert));
}

int floe_layer_build_table(const floe_layer* L, void* dev_table, size_t bytes, void* stream) {
    int rc = check_layer(L);
    if (rc) return rc;
    if (!L->experts || !dev_table || !aligned(dev_table, kAlign)) return FLOE_EINVAL;
    if (bytes < floe_layer_table_bytes(L)) return FLOE_EWORKSPACE;
    const int n = L->n_experts + L->n_shared;
    std::vector<DevExpert> host(n);
    for (int i = 0; i < n; ++i) {
        const floe_expert& e = L->experts[i];
        if (e.s.d != L->s.d || e.s.f != L->s.f || e.s.bits != L->s.bits || e.s.group != L->s.group) return FLOE_ESHAPE;
        if (!e.up_codes || !e.up_scale || !e.up_zero || !e.gd) return FLOE_EINVAL;
        // the batch kernels fetch scales and zeros with 16-byte loads: checked here, once, for every expert, so that
        // no decode call has to look at the host array again
        if (!aligned(e.up_codes, 16) || !aligned(e.gd, 16) || !aligned(e.up_scale, 16) || !aligned(e.up_zero, 16))
            return FLOE_EINVAL;
        if (e.gd_is_staged || e.gd_rows != e.s.f) return FLOE_EINVAL;
        host[i].codes = e.up_codes;
        host[i].scale = reinterpret_cast<const h16*>(e.up_scale);
        host[i].zero = reinterpret_cast<const h16*>(e.up_zero);
        host[i].gd = reinterpret_cast<const h16*>(e.gd);
        if (L->gd_on_host) {  // the kernels read pinned host memory through its device-side address
            void* dev_view = nullptr;
            FLOE_HIP(hipHostGetDevicePointer(&dev_view, const_cast<floe_half*>(e.gd), 0));
            host[i].gd = static_cast<const h16*>(dev_view);
        }
    }
    hipStream_t st = (hipStream_t)stream;
    FLOE_HIP(hipMemcpyAsync(dev_table, host.data(), (size_t)n * sizeof(DevExpert), hipMemcpyHostToDevice, st));
    FLOE_HIP(hipStreamSynchronize(st));
    return FLOE_OK;
}

size_t floe_layer_workspace_bytes(const floe_layer* L, int T) {
    if (check_layer(L) != FLOE_OK || T < 0) return 0;
    return layer_ws(L, T).total;
}

int floe_moe_layer_decode(const floe_layer* L, const floe_half* x, int T, floe_half* y, floe_slot_stat* stats,
                          void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_layer(L);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;
    if (!L->dev_table || !x || !y || !workspace) return FLOE_EINVAL;
    if (L->gd_on_host) return FLOE_EINVAL;  // host-resident gate/down: use floe_moe_layer_decode_offloaded
    if (!aligned(x, 16) || !aligned(y, 8) || !aligned(workspace, kAlign)) return FLOE_EINVAL;
    const LayerWs w = layer_ws(L, T);
    if (workspace_bytes < w.total) return FLOE_EWORKSPACE;
    char* base = static_cast<char*>(workspace);
    DevExpert* task_table = reinterpret_cast<DevExpert*>(base + w.table_off);
    int32_t* task_expert = reinterpret_cast<int32_t*>(base + w.expert_off);
    float* task_weight = reinterpret_cast<float*>(base + w.weight_off);
    float* task_tau = reinterpret_cast<float*>(base + w.tau_off);
    int32_t* count = reinterpret_cast<int32_t*>(base + w.count_off);
    uint32_t* mask = reinterpret_cast<uint32_t*>(base + w.mask_off);
    float* v = reinterpret_cast<float*>(base + w.v_off);
    int32_t* idx = reinterpret_cast<int32_t*>(base + w.idx_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = (hipStream_t)stream;
    const h16* xh = reinterpret_cast<const h16*>(x);
    const int slots = L->top_k + L->n_shared;

    TaskMap map{};
    map.task_table = task_table;
    map.slots = slots;
    const bool mask_ok = mask_path_ok(L->s.f);
    const bool batch_mfma = w.batch_mfma;
    int nblk = w.nblk, count_parts = 0;
    if (w.fused_passes && !batch_mfma) {
        // small batch: [(router +) up GEMV + selection + gate/down on the workgroup's own channels] -> [combine];
        // with <= 16 experts the router runs inside the same kernel; with <= 64 its dot products run in a kernel in front
        // and softmax / top-k inside; otherwise the whole router runs in front
        const int route_mode = fused_route_mode(L->n_experts, L->top_k, L->n_shared);
        const bool in_place = route_mode != 0;
        RouteArgs ro{};
        ro.router_cm = reinterpret_cast<const h16*>(L->router_cm);
        ro.tau = L->tau;
        ro.tau_stride_t = L->tau_stride_t;
        ro.n_experts = L->n_experts; ro.top_k = L->top_k; ro.n_shared = L->n_shared; ro.renormalize = L->renormalize;
        ro.table = static_cast<const DevExpert*>(L->dev_table);
        ro.task_table = task_table;
        ro.task_expert = task_expert; ro.task_weight = task_weight; ro.task_tau = task_tau;
        if (route_mode == 0) {
            const RouterArgs ra = router_args(L, w, base, xh);
            FLOE_LAUNCH(FLOE_KERNEL_ROUTER, st, launch_router(ra, T, st));
        } else if (route_mode == 1) {
            const RouterArgs ra = router_args(L, w, base, xh);
            if (!ra.logits) return FLOE_EWORKSPACE;
            FLOE_LAUNCH(FLOE_KERNEL_ROUTER, st, launch_router_logits(ra, T, st));
            ro.logits = ra.logits;
        }
        FusedArgs a{};
        a.map = map; a.x = xh; a.route = in_place ? &ro : nullptr; a.task_tau = task_tau; a.task_scale = task_weight;
        a.v_out = nullptr; a.partial = partial; a.wg_count = count;
        a.d = L->s.d; a.f = L->s.f; a.group = L->s.group; a.n_tasks = w.n_tasks; a.passes = w.fused_passes;
        FLOE_LAUNCH(FLOE_KERNEL_FUSED_FFN, st, launch_fused(a, L->s.bits, st));
        nblk = w.nblk_fused;
        count_parts = w.nblk_fused;
    } else if (w.use_union) {
        // decode batch: [router] -> [token groups per expert] -> [up GEMV + mask bits] -> [gate on the union of the
        // group's rows] -> [down]; every selected row is read once per expert group
        const RouterArgs ra = router_args(L, w, base, xh);
        FLOE_LAUNCH(FLOE_KERNEL_ROUTER, st, launch_router(ra, T, st));
        TokenGroup* groups = reinterpret_cast<TokenGroup*>(base + w.groups_off);
        int32_t* n_groups = reinterpret_cast<int32_t*>(base + w.ngroups_off);
        const int n_all = L->n_experts + L->n_shared;
        FLOE_HIP(launch_group_tokens(task_expert, w.n_tasks, n_all, w.chunk, groups, n_groups, st));
        if (batch_mfma)
            FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                        launch_up_gemv_grouped(static_cast<const DevExpert*>(L->dev_table), groups, n_groups,
                                               w.up.max_groups, w.chunk, xh, slots, v, task_tau, mask, L->s.d, L->s.f,
                                               L->s.bits, L->s.group, st));
        else
            FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                        launch_up_gemv(map, xh, nullptr, v, task_tau, mask, L->s.d, L->s.f, L->s.bits, L->s.group,
                                       w.n_tasks, st));
        UnionArgs ua{};
        ua.table = static_cast<const DevExpert*>(L->dev_table);
        ua.groups = groups; ua.n_groups = n_groups; ua.x = xh; ua.v = v; ua.mask_words = mask;
        ua.task_scale = task_weight; ua.count = count; ua.partial = partial;
        ua.urow = reinterpret_cast<int32_t*>(base + w.urow_off);
        ua.ucount = reinterpret_cast<int32_t*>(base + w.ucount_off);
        ua.hbuf = reinterpret_cast<uint4*>(base + w.hbuf_off);
        ua.slots = slots; ua.f = L->s.f; ua.nt = w.up.nt; ua.cap = w.up.cap;
        ua.nblk_gate = w.up.nblk_gate; ua.nblk_down = w.up.nblk_down;
        FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st, launch_gate_down_union(ua, w.up, L->s.d, st));
        nblk = w.up.nblk_down;
        count_parts = w.up.nblk_gate;
    } else if (mask_ok && !batch_mfma &&
               route_in_place_ok(L->s.d, L->s.bits, L->s.group, L->n_experts, L->top_k, L->n_shared)) {
        // larger batches of shapes without a matrix-core path: [router + up GEMV + mask] -> [compaction + gate/down]
        RouteArgs ro{};
        ro.router_cm = reinterpret_cast<const h16*>(L->router_cm);
        ro.tau = L->tau;
        ro.tau_stride_t = L->tau_stride_t;
        ro.n_experts = L->n_experts; ro.top_k = L->top_k; ro.n_shared = L->n_shared; ro.renormalize = L->renormalize;
        ro.table = static_cast<const DevExpert*>(L->dev_table);
        ro.task_table = task_table;
        ro.task_expert = task_expert; ro.task_weight = task_weight; ro.task_tau = task_tau;
        FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                    launch_up_gemv(map, xh, &ro, v, nullptr, mask, L->s.d, L->s.f, L->s.bits, L->s.group,
                                   w.n_tasks, st));
        FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                    launch_gate_down(map, nullptr, L->s.f, xh, v, mask, nullptr, count, task_weight, partial, L->s.d, L->s.f,
                                     w.n_tasks, w.nblk, st));
    } else {
        const RouterArgs ra = router_args(L, w, base, xh);
        FLOE_LAUNCH(FLOE_KERNEL_ROUTER, st, launch_router(ra, T, st));
        // batches: the gate/down workgroups are launched in expert order (tasks that share an expert run side by side
        // and share its rows in the L2)
        TokenGroup* groups = reinterpret_cast<TokenGroup*>(base + w.groups_off);
        int32_t* n_groups = reinterpret_cast<int32_t*>(base + w.ngroups_off);
        // (only where the grouping kernel runs anyway: on its own it costs what the sharing saves)
        int32_t* order = (mask_ok && batch_mfma && w.n_tasks > kExpertOrderTasks) ? reinterpret_cast<int32_t*>(base + w.order_off) : nullptr;
        const int n_all = L->n_experts + L->n_shared;
        const int chunk = mfma_chunk(n_all, w.n_tasks);
        if (order || (mask_ok && batch_mfma))
            FLOE_HIP(launch_group_tokens(task_expert, w.n_tasks, n_all, chunk, groups, n_groups, st, order));
        if (mask_ok && batch_mfma) {
            // decode batch: tokens routed to the same expert share one pass over its codes (matrix cores)
            FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                        launch_up_gemv_grouped(static_cast<const DevExpert*>(L->dev_table), groups, n_groups,
                                               mfma_max_groups(n_all, w.n_tasks), chunk, xh, slots, v, task_tau,
                                               mask, L->s.d, L->s.f, L->s.bits, L->s.group, st));
            FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                        launch_gate_down(map, nullptr, L->s.f, xh, v, mask, nullptr, count, task_weight, partial, L->s.d,
                                         L->s.f, w.n_tasks, w.nblk, st, nullptr, order));
        } else if (mask_ok) {
            FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                        launch_up_gemv(map, xh, nullptr, v, task_tau, mask, L->s.d, L->s.f, L->s.bits, L->s.group,
                                       w.n_tasks, st));
            FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                        launch_gate_down(map, nullptr, L->s.f, xh, v, mask, nullptr, count, task_weight, partial, L->s.d,
                                         L->s.f, w.n_tasks, w.nblk, st, nullptr, order));
        } else {
            FLOE_LAUNCH(FLOE_KERNEL_UP_GEMV, st,
                        launch_up_gemv(map, xh, nullptr, v, nullptr, nullptr, L->s.d, L->s.f, L->s.bits,
                                       L->s.group, w.n_tasks, st));
            FLOE_LAUNCH(FLOE_KERNEL_SELECT, st, launch_select(v, L->s.f, w.n_tasks, task_tau, idx, count, st));
            FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                        launch_gate_down(map, nullptr, L->s.f, xh, v, nullptr, idx, count, task_weight, partial, L->s.d,
                                         L->s.f, w.n_tasks, w.nblk, st));
        }
    }
    FLOE_LAUNCH(FLOE_KERNEL_COMBINE, st, launch_combine(partial, L->s.d, T, slots, nblk, nullptr, reinterpret_cast<h16*>(y), st));
    if (stats)
        FLOE_HIP(launch_stats(task_expert, count, count_parts, task_weight, reinterpret_cast<SlotStat*>(stats), w.n_tasks, st));
    return FLOE_OK;
}

int floe_moe_layer_decode_offloaded(const floe_layer* L, const floe_offload* o, const floe_half* x, int T, floe_half* y,
                                    floe_slot_stat* stats, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_layer(L);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;
    if (!o || !o->staging || !o->ev_lists_ready || !o->ev_staged || o->capacity_rows <= 0) return FLOE_EINVAL;
    if (!L->dev_table || !L->gd_on_host || !x || !y || !workspace) return FLOE_EINVAL;
    if (!aligned(x, 16) || !aligned(y, 8) || !aligned(workspace, kAlign) || !aligned(o->staging, 16)) return FLOE_EINVAL;
    const LayerWs w = layer_ws(L, T);
    if (workspace_bytes < w.total) return FLOE_EWORKSPACE;
    char* base = static_cast<char*>(workspace);
    DevExpert* task_table = reinterpret_cast<DevExpert*>(base + w.table_off);
    int32_t* task_expert = reinterpret_cast<int32_t*>(base + w.expert_off);
    float* task_weight = reinterpret_cast<float*>(base + w.weight_off);
    int32_t* count = reinterpret_cast<int32_t*>(base + w.count_off);
    float* v = reinterpret_cast<float*>(base + w.v_off);
    int32_t* idx = reinterpret_cast<int32_t*>(base + w.idx_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = (hipStream_t)stream, side = (hipStream_t)o->side_stream;
    const h16* xh = reinterpret_cast<const h16*>(x);
    const int slots = L->top_k + L->n_shared;

    TaskMap map{};
    map.task_table = task_table;
    map.slots = slots;
    if ((rc = layer_lists(L, w, base, xh, T, st))) return rc;
    FLOE_HIP(hipEventRecord((hipEvent_t)o->ev_lists_ready, st));
    FLOE_HIP(hipStreamWaitEvent(side, (hipEvent_t)o->ev_lists_ready, 0));
    FLOE_LAUNCH(FLOE_KERNEL_STAGE, side,
                launch_stage_tasks(task_table, L->s.d, L->s.f, idx, count, o->capacity_rows,
                                   reinterpret_cast<h16*>(o->staging), o->overflow, w.n_tasks, side));
    FLOE_HIP(hipEventRecord((hipEvent_t)o->ev_staged, side));
    FLOE_HIP(hipStreamWaitEvent(st, (hipEvent_t)o->ev_staged, 0));
    FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                launch_gate_down(map, reinterpret_cast<const h16*>(o->staging), o->capacity_rows, xh, v, nullptr, idx,
                                 count, task_weight, partial, L->s.d, L->s.f, w.n_tasks, w.nblk, st));
    FLOE_LAUNCH(FLOE_KERNEL_COMBINE, st,
                launch_combine(partial, L->s.d, T, slots, w.nblk, nullptr, reinterpret_cast<h16*>(y), st));
    if (stats)
        FLOE_HIP(launch_stats(task_expert, count, 0, task_weight, reinterpret_cast<SlotStat*>(stats), w.n_tasks, st, count,
                              o->capacity_rows));
    return FLOE_OK;
}

int floe_moe_layer_prefetch(const floe_layer* L, const floe_prefetch* p, const floe_half* x_cur, int T, void* workspace,
                            size_t workspace_bytes, void* stream) {
    int rc = check_layer(L);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;
    if (!p || !p->staging || !p->pred_expert || !p->pred_count || !p->row_of || !p->ev_inputs_ready || !p->ev_prefetched ||
        p->capacity_rows <= 0)
        return FLOE_EINVAL;
    if (!L->dev_table || !L->gd_on_host || !x_cur || !workspace) return FLOE_EINVAL;
    if (!aligned(x_cur, 16) || !aligned(workspace, kAlign) || !aligned(p->staging, 16)) return FLOE_EINVAL;
    const LayerWs w = layer_ws(L, T);
    if (workspace_bytes < w.total) return FLOE_EWORKSPACE;
    char* base = static_cast<char*>(workspace);
    hipStream_t st = (hipStream_t)stream, side = (hipStream_t)p->prefetch_stream;
    // everything below runs on the prefetch stream, after whatever produced x_cur on `stream`
    FLOE_HIP(hipEventRecord((hipEvent_t)p->ev_inputs_ready, st));
    FLOE_HIP(hipStreamWaitEvent(side, (hipEvent_t)p->ev_inputs_ready, 0));
    if ((rc = layer_lists(L, w, base, reinterpret_cast<const h16*>(x_cur), T, side))) return rc;
    const DevExpert* task_table = reinterpret_cast<const DevExpert*>(base + w.table_off);
    const int32_t* task_expert = reinterpret_cast<const int32_t*>(base + w.expert_off);
    const int32_t* count = reinterpret_cast<const int32_t*>(base + w.count_off);
    const int32_t* idx = reinterpret_cast<const int32_t*>(base + w.idx_off);
    FLOE_LAUNCH(FLOE_KERNEL_STAGE, side,
                launch_stage_tasks(task_table, L->s.d, L->s.f, idx, count, p->capacity_rows,
                                   reinterpret_cast<h16*>(p->staging), nullptr, w.n_tasks, side));
    FLOE_HIP(launch_rowmap(idx, count, task_expert, L->s.f, p->capacity_rows, p->row_of, p->pred_expert, p->pred_count,
                           w.n_tasks, side));
    FLOE_HIP(hipEventRecord((hipEvent_t)p->ev_prefetched, side));
    return FLOE_OK;
}

int floe_moe_layer_decode_prefetched(const floe_layer* L, const floe_prefetch* p, const floe_miss_path* m,
                                     const floe_half* x, int T, floe_half* y, floe_slot_stat* stats,
                                     floe_prefetch_stat* prefetch_stats, void* workspace, size_t workspace_bytes,
                                     void* stream) {
    static_assert(sizeof(floe_prefetch_stat) == sizeof(PrefetchStat), "prefetch stat record layout");
    int rc = check_layer(L);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;
    if (!p || !p->staging || !p->pred_expert || !p->pred_count || !p->row_of || !p->ev_prefetched || p->capacity_rows <= 0)
        return FLOE_EINVAL;
    if (!m || !m->ev_lists_ready || !m->ev_staged) return FLOE_EINVAL;
    if (!L->dev_table || !L->gd_on_host || !x || !y || !workspace) return FLOE_EINVAL;
    if (!aligned(x, 16) || !aligned(y, 8) || !aligned(workspace, kAlign) || !aligned(p->staging, 16)) return FLOE_EINVAL;
    const LayerWs w = layer_ws(L, T);
    if (workspace_bytes < w.total) return FLOE_EWORKSPACE;
    char* base = static_cast<char*>(workspace);
    DevExpert* task_table = reinterpret_cast<DevExpert*>(base + w.table_off);
    int32_t* task_expert = reinterpret_cast<int32_t*>(base + w.expert_off);
    float* task_weight = reinterpret_cast<float*>(base + w.weight_off);
    int32_t* count = reinterpret_cast<int32_t*>(base + w.count_off);
    float* v = reinterpret_cast<float*>(base + w.v_off);
    int32_t* idx = reinterpret_cast<int32_t*>(base + w.idx_off);
    int32_t* rows = reinterpret_cast<int32_t*>(base + w.rows_off);
    int32_t* miss_idx = reinterpret_cast<int32_t*>(base + w.missidx_off);
    int32_t* miss_rows = reinterpret_cast<int32_t*>(base + w.missrows_off);
    int32_t* miss_count = reinterpret_cast<int32_t*>(base + w.misscount_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = (hipStream_t)stream, side = (hipStream_t)m->miss_stream;
    const h16* xh = reinterpret_cast<const h16*>(x);
    const int slots = L->top_k + L->n_shared;
    TaskMap map{};
    map.task_table = task_table;
    map.slots = slots;

    if ((rc = layer_lists(L, w, base, xh, T, st))) return rc;
    FLOE_HIP(hipStreamWaitEvent(st, (hipEvent_t)p->ev_prefetched, 0));
    FLOE_HIP(launch_match_rows(idx, count, task_expert, L->s.f, slots, p->capacity_rows, p->row_of, p->pred_expert,
                               p->pred_count, rows, miss_idx, miss_rows, miss_count, m->overflow,
                               reinterpret_cast<PrefetchStat*>(prefetch_stats), w.n_tasks, st));
    FLOE_HIP(hipEventRecord((hipEvent_t)m->ev_lists_ready, st));
    FLOE_HIP(hipStreamWaitEvent(side, (hipEvent_t)m->ev_lists_ready, 0));
    FLOE_LAUNCH(FLOE_KERNEL_STAGE, side,
                launch_stage_tasks(task_table, L->s.d, L->s.f, miss_idx, miss_count, p->capacity_rows,
                                   reinterpret_cast<h16*>(p->staging), nullptr, w.n_tasks, side, miss_rows));
    FLOE_HIP(hipEventRecord((hipEvent_t)m->ev_staged, side));
    FLOE_HIP(hipStreamWaitEvent(st, (hipEvent_t)m->ev_staged, 0));
    FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                launch_gate_down(map, reinterpret_cast<const h16*>(p->staging), p->capacity_rows, xh, v, nullptr, idx, count,
                                 task_weight, partial, L->s.d, L->s.f, w.n_tasks, w.nblk, st, rows));
    FLOE_LAUNCH(FLOE_KERNEL_COMBINE, st,
                launch_combine(partial, L->s.d, T, slots, w.nblk, nullptr, reinterpret_cast<h16*>(y), st));
    if (stats)
        FLOE_HIP(launch_stats(task_expert, count, 0, task_weight, reinterpret_cast<SlotStat*>(stats), w.n_tasks, st, miss_count));
    return FLOE_OK;
}

int floe_channel_cache_load(const floe_layer* L, const floe_channel_cache* c, int expert, const int32_t* idx,
                            const int32_t* count, int first_row, int max_rows, void* stream) {
    int rc = check_layer(L);
    if (rc) return rc;
    if (!c || !c->pool || !c->row_of || !idx || !count || !L->dev_table || !L->gd_on_host) return FLOE_EINVAL;
    if (expert < 0 || expert >= L->n_experts + L->n_shared || first_row < 0 || max_rows < 0) return FLOE_EINVAL;
    if ((long long)first_row + max_rows > c->resident_rows) return FLOE_EINVAL;  // the resident part of the pool ends there
    if (!aligned(c->pool, 16)) return FLOE_EINVAL;
    FLOE_LAUNCH(FLOE_KERNEL_STAGE, (hipStream_t)stream,
                launch_cache_load(static_cast<const DevExpert*>(L->dev_table), expert, L->s.d, L->s.f, idx, count, first_row,
                                  max_rows, reinterpret_cast<h16*>(c->pool), c->row_of, (hipStream_t)stream));
    return FLOE_OK;
}

int floe_moe_layer_decode_cached(const floe_layer* L, const floe_channel_cache* c, const floe_miss_path* m,
                                 const floe_half* x, int T, floe_half* y, floe_slot_stat* stats,
                                 floe_prefetch_stat* cache_stats, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_layer(L);
    if (rc) return rc;
    if ((rc = check_T(T))) return rc;
    if (T == 0) return FLOE_OK;
    if (!c || !c->pool || !c->row_of || c->capacity_rows <= 0 || c->resident_rows < 0) return FLOE_EINVAL;
    if (!m || !m->ev_lists_ready || !m->ev_staged) return FLOE_EINVAL;
    if (!L->dev_table || !L->gd_on_host || !x || !y || !workspace) return FLOE_EINVAL;
    if (!aligned(x, 16) || !aligned(y, 8) || !aligned(workspace, kAlign) || !aligned(c->pool, 16)) return FLOE_EINVAL;
    const LayerWs w = layer_ws(L, T);
    if (workspace_bytes < w.total) return FLOE_EWORKSPACE;
    char* base = static_cast<char*>(workspace);
    DevExpert* task_table = reinterpret_cast<DevExpert*>(base + w.table_off);
    int32_t* task_expert = reinterpret_cast<int32_t*>(base + w.expert_off);
    float* task_weight = reinterpret_cast<float*>(base + w.weight_off);
    int32_t* count = reinterpret_cast<int32_t*>(base + w.count_off);
    float* v = reinterpret_cast<float*>(base + w.v_off);
    int32_t* idx = reinterpret_cast<int32_t*>(base + w.idx_off);
    int32_t* rows = reinterpret_cast<int32_t*>(base + w.rows_off);
    int32_t* miss_idx = reinterpret_cast<int32_t*>(base + w.missidx_off);
    int32_t* miss_rows = reinterpret_cast<int32_t*>(base + w.missrows_off);
    int32_t* miss_count = reinterpret_cast<int32_t*>(base + w.misscount_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = (hipStream_t)stream, side = (hipStream_t)m->miss_stream;
    const h16* xh = reinterpret_cast<const h16*>(x);
    const int slots = L->top_k + L->n_shared;
    TaskMap map{};
    map.task_table = task_table;
    map.slots = slots;

    // lists on `stream`; where each selected channel sits (resident row, or a fresh row of the task's slab) and which
    // ones are missing; the misses cross the bus on the miss stream; gate/down on the pool's rows
    if ((rc = layer_lists(L, w, base, xh, T, st))) return rc;
    FLOE_HIP(launch_match_rows(idx, count, task_expert, L->s.f, slots, c->capacity_rows, nullptr, nullptr, nullptr, rows,
                               miss_idx, miss_rows, miss_count, m->overflow, reinterpret_cast<PrefetchStat*>(cache_stats),
                               w.n_tasks, st, c->row_of, c->resident_rows));
    FLOE_HIP(hipEventRecord((hipEvent_t)m->ev_lists_ready, st));
    FLOE_HIP(hipStreamWaitEvent(side, (hipEvent_t)m->ev_lists_ready, 0));
    FLOE_LAUNCH(FLOE_KERNEL_STAGE, side,
                launch_stage_tasks(task_table, L->s.d, L->s.f, miss_idx, miss_count, c->capacity_rows,
                                   reinterpret_cast<h16*>(c->pool), nullptr, w.n_tasks, side, miss_rows));
    FLOE_HIP(hipEventRecord((hipEvent_t)m->ev_staged, side));
    FLOE_HIP(hipStreamWaitEvent(st, (hipEvent_t)m->ev_staged, 0));
    FLOE_LAUNCH(FLOE_KERNEL_GATE_DOWN, st,
                launch_gate_down(map, reinterpret_cast<const h16*>(c->pool), c->capacity_rows, xh, v, nullptr, idx, count,
                                 task_weight, partial, L->s.d, L->s.f, w.n_tasks, w.nblk, st, rows));
    FLOE_LAUNCH(FLOE_KERNEL_COMBINE, st,
                launch_combine(partial, L->s.d, T, slots, w.nblk, nullptr, reinterpret_cast<h16*>(y), st));
    if (stats)
        FLOE_HIP(launch_stats(task_expert, count, 0, task_weight, reinterpret_cast<SlotStat*>(stats), w.n_tasks, st, miss_count,
                              c->capacity_rows));
    return FLOE_OK;
}

int floe_stage_channels(const floe_half* host_gd, int d, int f, const int32_t* idx, const int32_t* count, int capacity_rows,
                        floe_half* hbm_dst, int32_t* overflow, void* side_stream, void* done) {
    if (!host_gd || !idx || !count || !hbm_dst) return FLOE_EINVAL;
    if (d <= 0 || f <= 0 || capacity_rows < 0) return FLOE_EINVAL;
    if (d % 4 != 0) return FLOE_ESHAPE;
    if (!aligned(host_gd, 16) || !aligned(hbm_dst, 16)) return FLOE_EINVAL;
    // the device view of the pinned matrix; callers stage from the same few matrices over and over
    static thread_local const floe_half* last_host = nullptr;
    static thread_local void* last_dev = nullptr;
    if (host_gd != last_host) {
        void* dev_view = nullptr;
        FLOE_HIP(hipHostGetDevicePointer(&dev_view, const_cast<floe_half*>(host_gd), 0));
        last_host = host_gd;
        last_dev = dev_view;
    }
    void* dev_view = last_dev;
    hipStream_t st = (hipStream_t)side_stream;
    FLOE_LAUNCH(FLOE_KERNEL_STAGE, st, launch_stage(static_cast<const h16*>(dev_view), d, f, idx, count, capacity_rows,
                          reinterpret_cast<h16*>(hbm_dst), overflow, st));
    if (done) FLOE_HIP(hipEventRecord((hipEvent_t)done, st));
    return FLOE_OK;
}

}  // extern "C"
