// Status/version queries, workspace sizing, the fused per-layer decode step, and the host-only
// retention-schedule helpers (Sec. 3.2, Eq. 7-9, Alg. 1 of the paper).
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "st3_evict.h"

namespace st3 {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

DebugState& debug_state() {
    static DebugState st = [] {
        const char* e = std::getenv("ST3_DEBUG");
        return DebugState{e != nullptr && std::strcmp(e, "1") == 0, 0, 0};
    }();
    return st;
}
static const bool g_debug_state_read_at_load = (debug_state(), true);

// ---------------------------------------------------------------------------------------------
// Optional timing of the decode attention kernel: a pool of hipEvent pairs attached to that
// kernel's launches (start and stop of the kernel itself).  Off unless st3_profile_enable().
// ---------------------------------------------------------------------------------------------
struct DecodeProfiler {
    std::mutex mu;
    std::vector<hipEvent_t> ev;     // 2 per launch
    size_t used = 0;                // launches recorded
    bool on = false;
};
static DecodeProfiler g_prof;

// Hands out the next event pair; the caller passes it to hipExtLaunchKernelGGL, which stamps the
// two events with the kernel's own start and end.
bool profile_take(hipEvent_t* start, hipEvent_t* stop) {
    if (!g_prof.on) return false;                   // (never set unless the debug block is enabled)
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (!g_prof.on) return false;
    if ((g_prof.used + 1) * 2 > g_prof.ev.size()) { g_prof.on = false; return false; }      // pool exhausted
    *start = g_prof.ev[g_prof.used * 2];
    *stop = g_prof.ev[g_prof.used * 2 + 1];
    g_prof.used += 1;
    return true;
}

st3_status validate_kv(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg);
st3_status validate_kv_value_only(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg);
st3_status enqueue_inherit(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                           int32_t max_kv_len, const void* v_new, const void* src_workspace,
                           size_t src_workspace_bytes, int32_t src_capacity, void* out, void* workspace,
                           size_t workspace_bytes, hipStream_t st, const PlanStash* stash = nullptr);
st3_status enqueue_decode(const st3_attn_shape* shape, const void* q, const st3_kv_layer* kv,
                          const st3_segments* seg, int32_t max_kv_len, const void* k_new, const void* v_new,
                          void* out, float* vis_mass, int64_t mass_stride, bool want_mass, bool defer_mass,
                          bool keep_all_logits, void* workspace, size_t workspace_bytes, hipStream_t st,
                          bool defer_merge = false, const PlanStash* stash = nullptr);
bool decode_is_split(const st3_attn_shape* shape, const st3_kv_layer* kv, int32_t max_kv_len);

}  // namespace st3

extern "C" const char* st3_status_string(st3_status s) {
    switch (s) {
        case ST3_OK: return "ok";
        case ST3_ERR_INVALID_ARG: return "invalid argument";
        case ST3_ERR_UNSUPPORTED: return "unsupported shape, type or size";
        case ST3_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case ST3_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

extern "C" int st3_last_hip_error(void) { return st3::g_last_hip_error; }
extern "C" uint32_t st3_version(void) { return (0u << 16) | (1u << 8) | 0u; }

extern "C" size_t st3_workspace_bytes(const st3_attn_shape* shape, int32_t kv_capacity, int32_t max_vis_len,
                                      int32_t score_window) {
    if (st3::check_shape(shape) != ST3_OK) return 0;
    if (kv_capacity < 0 || max_vis_len < 0) return 0;
    if (score_window < 1) score_window = 1;
    if (score_window > st3::kMaxWindow) score_window = st3::kMaxWindow;
    // decode region first, prefill scratch behind it: prefill never touches the pending-mass descriptors
    const size_t d = st3::decode_ws(shape->batch, shape->heads, shape->head_dim, kv_capacity).total;
    const size_t p = st3::prefill_ws(shape->batch, shape->heads, max_vis_len, score_window).total;
    return d + p;
}

namespace st3 {
__global__ void zero_i32_kernel(int32_t* p, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}
}  // namespace st3

extern "C" st3_status st3_workspace_init(const st3_attn_shape* shape, int32_t kv_capacity, void* workspace,
                                         size_t workspace_bytes, void* stream) {
    using namespace st3;
    st3_status s = check_shape(shape);
    if (s != ST3_OK) return s;
    if (!workspace || !aligned16(workspace) || kv_capacity <= 0) return ST3_ERR_INVALID_ARG;
    const DecodeWs wl = decode_ws(shape->batch, shape->heads, shape->head_dim, kv_capacity);
    if (workspace_bytes < wl.total) return ST3_ERR_WORKSPACE_TOO_SMALL;
    const int n = shape->batch * 4;
    zero_i32_kernel<<<(n + 255) / 256, 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(
        reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + wl.pending), n);
    return check_launch();
}

namespace st3 {
// Host-side checks of one layer's arguments for the fused step (shared by the per-layer and the
// whole-step entry points).
static st3_status check_layer_step(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                                   const float* score_col, const int32_t* id_col, int64_t col_stride,
                                   int32_t keep_after, int32_t mode, const void* q, const void* k_new,
                                   const void* v_new, const void* out, const float* vis_mass, int64_t mass_stride,
                                   const void* workspace, size_t workspace_bytes) {
    st3_status s = validate_kv(shape, kv, seg);
    if (s != ST3_OK) return s;
    if (!q || !k_new || !v_new || !out || !workspace) return ST3_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(workspace))
        return ST3_ERR_INVALID_ARG;
    if (seg->max_kv_len >= kv->capacity) return ST3_ERR_INVALID_ARG;
    if (vis_mass && mass_stride < seg->max_vis_len) return ST3_ERR_INVALID_ARG;
    if (keep_after >= 0) {
        if (!score_col || !id_col || col_stride < seg->max_vis_len) return ST3_ERR_INVALID_ARG;
        if (mode != ST3_STABLE && mode != ST3_HOLE_FILL) return ST3_ERR_INVALID_ARG;
    }
    const DecodeWs wl = decode_ws(shape->batch, shape->heads, shape->head_dim, kv->capacity);
    if (workspace_bytes < wl.total) return ST3_ERR_WORKSPACE_TOO_SMALL;
    return ST3_OK;
}

// A lazy layer of the whole-step call (Eq. 6, Alg. 2) against its source entry.
static st3_status check_lazy_step(const st3_attn_shape* shape, const st3_layer_step& L, const st3_layer_step& S,
                                  int32_t mode) {
    st3_status s = validate_kv_value_only(shape, &L.kv, &L.seg);
    if (s != ST3_OK) return s;
    if (S.inherit_from >= 0) return ST3_ERR_INVALID_ARG;                 // the source must attend by itself
    if (!L.v_new || !L.out || !L.workspace || !aligned16(L.v_new) || !aligned16(L.workspace))
        return ST3_ERR_INVALID_ARG;
    if (L.workspace == S.workspace) return ST3_ERR_INVALID_ARG;
    if (L.seg.max_kv_len >= L.kv.capacity) return ST3_ERR_INVALID_ARG;
    if (L.seg.sys_len != S.seg.sys_len || L.seg.max_vis_len != S.seg.max_vis_len ||
        L.seg.max_kv_len != S.seg.max_kv_len || L.keep_after != S.keep_after)
        return ST3_ERR_INVALID_ARG;                                      // both must hold and evict the same rows
    if (L.vis_mass && L.mass_stride < L.seg.max_vis_len) return ST3_ERR_INVALID_ARG;
    // the lazy layer's mass is finished from what the source's attend launch marks pending, and
    // that launch only does so when the source asks for its own mass
    if (L.vis_mass && !S.vis_mass) return ST3_ERR_INVALID_ARG;
    if (L.keep_after >= 0) {
        if (!L.score_col || !L.id_col || L.col_stride < L.seg.max_vis_len) return ST3_ERR_INVALID_ARG;
        if (L.score_col == S.score_col || L.id_col == S.id_col) return ST3_ERR_INVALID_ARG;  // own copies
        if (mode != ST3_STABLE && mode != ST3_HOLE_FILL) return ST3_ERR_INVALID_ARG;
    }
    const DecodeWs wl = decode_ws(shape->batch, shape->heads, shape->head_dim, L.kv.capacity);
    if (L.workspace_bytes < wl.total) return ST3_ERR_WORKSPACE_TOO_SMALL;
    return ST3_OK;
}

}  // namespace st3

extern "C" st3_status st3_decode_layer_step(const st3_attn_shape* shape, const st3_kv_layer* kv,
                                            const st3_segments* seg, float* score_col, int32_t* id_col,
                                            int64_t col_stride, int32_t keep_after, int32_t mode, const void* q,
                                            const void* k_new, const void* v_new, void* out, float* vis_mass,
                                            int64_t mass_stride, void* workspace, size_t workspace_bytes,
                                            void* stream) {
    using namespace st3;
    st3_status s = check_shape(shape);
    if (s != ST3_OK) return s;
    // all checks before the first launch, so that an error enqueues nothing
    s = check_layer_step(shape, kv, seg, score_col, id_col, col_stride, keep_after, mode, q, k_new, v_new, out,
                         vis_mass, mass_stride, workspace, workspace_bytes);
    if (s != ST3_OK) return s;
    EvictArgs ea;
    bool needs_apply = false;
    s = build_evict_args(shape, kv, seg, score_col, id_col, col_stride, keep_after, mode, workspace, workspace_bytes,
                         1, vis_mass, mass_stride, ea, needs_apply, false);
    if (s != ST3_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // (1) attention over the cache plus the new token, whose row is read from k_new/v_new and stored on the way
    s = enqueue_decode(shape, q, kv, seg, seg->max_kv_len + 1, k_new, v_new, out, vis_mass, mass_stride,
                       vis_mass != nullptr, true, false, workspace, workspace_bytes, st);
    if (s != ST3_OK) return s;
    // (2) one workgroup per sequence: finish the mass, count the appended row, rank and evict for the next step
    launch_evict_plan(ea, shape->batch, st);
    if (needs_apply) launch_evict_apply(ea, shape->batch, st);
    return check_launch();
}

namespace st3 {

// Host-side checks of every layer of a step and the eviction plans that go with them.  Nothing is
// enqueued here.  has_heirs[i]: some lazy layer inherits from layer i (its attend launch must then
// keep the logit of every key).
static st3_status check_step(const st3_attn_shape* shape, int32_t n_layers, const st3_layer_step* layers, int32_t mode,
                             std::vector<EvictArgs>& plan, std::vector<char>& needs_apply, std::vector<char>& has_heirs) {
    st3_status s = check_shape(shape);
    if (s != ST3_OK) return s;
    if (n_layers <= 0 || !layers) return ST3_ERR_INVALID_ARG;
    plan.assign((size_t)n_layers, EvictArgs{});
    needs_apply.assign((size_t)n_layers, 0);
    has_heirs.assign((size_t)n_layers, 0);
    for (int i = 0; i < n_layers; ++i)
        if (layers[i].inherit_from >= 0 && layers[i].inherit_from < i) has_heirs[layers[i].inherit_from] = 1;
    for (int i = 0; i < n_layers; ++i) {
        const st3_layer_step& L = layers[i];
        const bool lazy = L.inherit_from >= 0;
        if (lazy) {
            if (L.inherit_from >= i) return ST3_ERR_INVALID_ARG;
            s = check_lazy_step(shape, L, layers[L.inherit_from], mode);
        } else {
            s = check_layer_step(shape, &L.kv, &L.seg, L.score_col, L.id_col, L.col_stride, L.keep_after, mode, L.q,
                                 L.k_new, L.v_new, L.out, L.vis_mass, L.mass_stride, L.workspace, L.workspace_bytes);
        }
        if (s != ST3_OK) return s;
        bool na = false;
        // a lazy layer's mass is its source's: finished from the logits in the source's workspace
        const st3_layer_step* S = lazy ? &layers[L.inherit_from] : nullptr;
        s = build_evict_args(shape, &L.kv, &L.seg, L.score_col, L.id_col, L.col_stride, L.keep_after, mode,
                             L.workspace, L.workspace_bytes, 1, L.vis_mass, L.mass_stride, plan[i], na, true,
                             S ? S->workspace : nullptr, S ? S->kv.capacity : 0);
        if (s != ST3_OK) return s;
        needs_apply[i] = na ? 1 : 0;
    }
    return ST3_OK;
}

// Append + attention of layer i of a checked step; the mass stays pending for the layer's plan.
// merge_in_plan: strips cut into chunks leave their partials for the layer's plan to merge (the
// whole-step call); else a merge launch follows the attention and `out` is complete right after it.
// stash (may be null): words the launch leaves in the layer's workspace for the launch that plans the layer.
static st3_status enqueue_layer_attend(const st3_attn_shape* shape, const st3_layer_step* layers, int i, bool has_heirs,
                                       hipStream_t st, bool merge_in_plan, const PlanStash* stash = nullptr) {
    const st3_layer_step& L = layers[i];
    if (L.inherit_from >= 0) {
        const st3_layer_step& S = layers[L.inherit_from];
        return enqueue_inherit(shape, &L.kv, &L.seg, L.seg.max_kv_len + 1, L.v_new, S.workspace, S.workspace_bytes,
                               S.kv.capacity, L.out, L.workspace, L.workspace_bytes, st, stash);
    }
    return enqueue_decode(shape, L.q, &L.kv, &L.seg, L.seg.max_kv_len + 1, L.k_new, L.v_new, L.out, L.vis_mass,
                          L.mass_stride, L.vis_mass != nullptr, true, has_heirs, L.workspace, L.workspace_bytes, st,
                          merge_in_plan, stash);
}

// The plans of layers [i0, i1) (finish the mass, count the new row, rank, evict): a plan workgroup is
// latency bound, so the layers' plans are best run side by side.  Their arguments travel by value,
// 16 layers per launch, unless `stashed` tells where the layers' attention launches have left a copy
// of each plan in device memory: then one launch reads them there (up to 64 layers).
static void enqueue_plan_range(const std::vector<EvictArgs>& plan, const std::vector<char>& needs_apply, int i0, int i1,
                               int B, hipStream_t st, const std::vector<const EvictArgs*>* stashed = nullptr) {
    if (i1 <= i0) return;
    if (stashed != nullptr) launch_evict_plan_table(stashed->data() + i0, plan.data() + i0, i1 - i0, B, st);
    else launch_evict_plan_batch(plan.data() + i0, i1 - i0, B, st);
    for (int i = i0; i < i1; ++i)
        if (needs_apply[(size_t)i]) launch_evict_apply(plan[(size_t)i], B, st);
}

static st3_status enqueue_plans(const std::vector<EvictArgs>& plan, const std::vector<char>& needs_apply, int B,
                                hipStream_t st) {
    enqueue_plan_range(plan, needs_apply, 0, (int)plan.size(), B, st);
    return check_launch();
}

}  // namespace st3

extern "C" st3_status st3_decode_layer_attend(const st3_attn_shape* shape, int32_t n_layers, const st3_layer_step* layers,
                                              int32_t layer, int32_t mode, void* stream) {
    using namespace st3;
    st3_status s = check_shape(shape);
    if (s != ST3_OK) return s;
    if (n_layers <= 0 || !layers || layer < 0 || layer >= n_layers) return ST3_ERR_INVALID_ARG;
    // only this layer's entry (and its source's) is checked here; st3_decode_plans checks the whole array
    const st3_layer_step& L = layers[layer];
    if (L.inherit_from >= 0) {
        if (L.inherit_from >= layer) return ST3_ERR_INVALID_ARG;
        s = check_lazy_step(shape, L, layers[L.inherit_from], mode);
    } else {
        s = check_layer_step(shape, &L.kv, &L.seg, L.score_col, L.id_col, L.col_stride, L.keep_after, mode, L.q, L.k_new,
                             L.v_new, L.out, L.vis_mass, L.mass_stride, L.workspace, L.workspace_bytes);
    }
    if (s != ST3_OK) return s;
    bool has_heirs = false;
    for (int i = layer + 1; i < n_layers; ++i) has_heirs = has_heirs || layers[i].inherit_from == layer;
    return enqueue_layer_attend(shape, layers, layer, has_heirs, reinterpret_cast<hipStream_t>(stream), false);
}

extern "C" st3_status st3_decode_plans(const st3_attn_shape* shape, int32_t n_layers, const st3_layer_step* layers,
                                       int32_t mode, void* stream) {
    using namespace st3;
    std::vector<EvictArgs> plan;
    std::vector<char> needs_apply, has_heirs;
    st3_status s = check_step(shape, n_layers, layers, mode, plan, needs_apply, has_heirs);
    if (s != ST3_OK) return s;
    return enqueue_plans(plan, needs_apply, shape->batch, reinterpret_cast<hipStream_t>(stream));
}

extern "C" st3_status st3_decode_step(const st3_attn_shape* shape, int32_t n_layers, const st3_layer_step* layers,
                                      int32_t mode, void* stream) {
    using namespace st3;
    std::vector<EvictArgs> plan;
    std::vector<char> needs_apply, has_heirs;
    st3_status s = check_step(shape, n_layers, layers, mode, plan, needs_apply, has_heirs);
    if (s != ST3_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // All of a step's inputs are here, so nothing needs a layer's output before the step ends: where
    // the strips are cut into chunks (B*H alone does not fill the chip) the chunk partials are merged
    // by the layer's plan instead of by a launch of their own behind every attention.
    std::vector<const EvictArgs*> stashed((size_t)n_layers, nullptr);
    for (int i = 0; i < n_layers; ++i) {
        const st3_layer_step& L = layers[i];
        const bool in_plan = L.inherit_from < 0 && decode_is_split(shape, &L.kv, L.seg.max_kv_len + 1);
        if (in_plan) {
            const DecodeWs wl = decode_ws(shape->batch, shape->heads, shape->head_dim, L.kv.capacity);
            char* ws = reinterpret_cast<char*>(L.workspace);
            plan[i].merge_part_o = reinterpret_cast<const float*>(ws + wl.part_o);
            plan[i].merge_out = L.out;
            plan[i].merge_D = shape->head_dim;
            plan[i].merge_bf16 = shape->dtype == ST3_BF16 ? 1 : 0;
            plan[i].part_ml = reinterpret_cast<const float*>(ws + wl.part_ml);
            plan[i].pending = reinterpret_cast<const int32_t*>(ws + wl.pending);
            plan[i].nsplit_cap = wl.nsplit_cap;
        }
        // the layer's plan travels with its attention launch into the layer's workspace; the plan launches read it there
        PlanStash stash{};
        std::memcpy(stash.w, &plan[i], sizeof(EvictArgs));
        {
            const DecodeWs wl = decode_ws(shape->batch, shape->heads, shape->head_dim, L.kv.capacity);
            stash.dst = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(L.workspace) + wl.plan_args);
            stashed[i] = reinterpret_cast<const EvictArgs*>(stash.dst);
        }
        s = enqueue_layer_attend(shape, layers, i, has_heirs[i] != 0, st, in_plan, &stash);
        if (s != ST3_OK) return s;
    }
    enqueue_plan_range(plan, needs_apply, 0, n_layers, shape->batch, st, &stashed);
    return check_launch();
}

extern "C" st3_status st3_profile_enable(int32_t max_launches) {
    using namespace st3;
    if (!debug_state().enabled) return ST3_ERR_UNSUPPORTED;
    if (max_launches <= 0 || max_launches > (1 << 22)) return ST3_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    while (g_prof.ev.size() < (size_t)max_launches * 2) {
        hipEvent_t e;
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) { set_last_hip_error(err); return ST3_ERR_HIP; }
        g_prof.ev.push_back(e);
    }
    g_prof.used = 0;
    g_prof.on = true;
    return ST3_OK;
}

extern "C" st3_status st3_profile_read(double* total_ms, int64_t* launches, double* min_ms, double* max_ms) {
    using namespace st3;
    if (!debug_state().enabled) return ST3_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    g_prof.on = false;
    double tot = 0.0, mn = 1e30, mx = 0.0;
    for (size_t i = 0; i < g_prof.used; ++i) {
        hipError_t err = hipEventSynchronize(g_prof.ev[2 * i + 1]);
        float ms = 0.f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]);
        if (err != hipSuccess) { set_last_hip_error(err); return ST3_ERR_HIP; }
        tot += ms; mn = ms < mn ? ms : mn; mx = ms > mx ? ms : mx;
    }
    if (total_ms) *total_ms = tot;
    if (launches) *launches = (int64_t)g_prof.used;
    if (min_ms) *min_ms = g_prof.used ? mn : 0.0;
    if (max_ms) *max_ms = mx;
    g_prof.used = 0;
    return ST3_OK;
}

extern "C" int st3_debug_enabled(void) { return st3::debug_state().enabled ? 1 : 0; }

extern "C" st3_status st3_debug_set_prefill_path(int path) {
    if (!st3::debug_state().enabled) return ST3_ERR_UNSUPPORTED;
    if (path < 0 || path > 2) return ST3_ERR_INVALID_ARG;
    st3::debug_state().prefill_path = path;
    return ST3_OK;
}

extern "C" st3_status st3_debug_set_attend_tile(int tile_loads) {
    if (!st3::debug_state().enabled) return ST3_ERR_UNSUPPORTED;
    st3::debug_state().attend_tile = tile_loads < 0 ? 0 : tile_loads;
    return ST3_OK;
}

// ---------------------------------------------------------------------------------------------
// Retention schedules (host only)
// ---------------------------------------------------------------------------------------------
extern "C" st3_status st3_schedule_pvtp(int32_t L, int32_t n_vis, int32_t first_layer, int32_t stride_S,
                                        int32_t P_bp, int32_t R_bp, int32_t* keep_l) {
    if (!keep_l || L <= 0 || n_vis < 0 || first_layer < 0 || stride_S <= 0) return ST3_ERR_INVALID_ARG;
    if (P_bp < 0 || P_bp > 10000 || R_bp < 0 || R_bp > 10000) return ST3_ERR_INVALID_ARG;
    int64_t gone_bp = 0;            // share of the ORIGINAL count removed so far
    for (int32_t l = 0; l < L; ++l) {
        if (l == first_layer) gone_bp += P_bp;
        else if (l > first_layer && (l - first_layer) % stride_S == 0) gone_bp += R_bp;
        int64_t left_bp = gone_bp >= 10000 ? 0 : 10000 - gone_bp;
        keep_l[l] = (int32_t)(((int64_t)n_vis * left_bp) / 10000);
    }
    return ST3_OK;
}

extern "C" st3_status st3_schedule_linear(int32_t L, int32_t n_vis, int32_t last_full_layer, int32_t end_ratio_bp,
                                          int32_t* keep_l) {
    if (!keep_l || L <= 0 || n_vis < 0 || last_full_layer < 0) return ST3_ERR_INVALID_ARG;
    if (end_ratio_bp < 0 || end_ratio_bp > 10000) return ST3_ERR_INVALID_ARG;
    const int64_t span = (int64_t)(L - 1) - last_full_layer;
    for (int32_t l = 0; l < L; ++l) {
        if (l <= last_full_layer || span <= 0) { keep_l[l] = n_vis; continue; }
        const int64_t num = (int64_t)n_vis * (10000 - end_ratio_bp) * (l - last_full_layer);
        const int64_t den = 10000 * span;
        keep_l[l] = (int32_t)(n_vis - (num + den - 1) / den);       // dropped count rounded up
    }
    return ST3_OK;
}

extern "C" st3_status st3_schedule_anneal(int32_t kind, double param, int32_t T, const int32_t* keep_l0, int32_t L,
                                          int32_t* keep_lt) {
    if (!keep_l0 || !keep_lt || L <= 0 || T < 0) return ST3_ERR_INVALID_ARG;
    if (kind < ST3_ANNEAL_COS || kind > ST3_ANNEAL_NONE) return ST3_ERR_INVALID_ARG;
    if (kind != ST3_ANNEAL_NONE && kind != ST3_ANNEAL_DROP && !(param > 0.0)) return ST3_ERR_INVALID_ARG;
    const double half_pi = 1.57079632679489661923;
    for (int32_t l = 0; l < L; ++l) {
        const int32_t k0 = keep_l0[l];
        if (k0 < 0) return ST3_ERR_INVALID_ARG;
        for (int32_t t = 0; t <= T; ++t) {
            int64_t c;
            switch (kind) {
                case ST3_ANNEAL_COS:
                    c = t < param ? (int64_t)std::floor(k0 * std::cos(t * half_pi / param) + 1e-9) : 0; break;
                case ST3_ANNEAL_LINEAR:
                    c = t < param ? (int64_t)std::floor(k0 * (1.0 - t / param) + 1e-9) : 0; break;
                case ST3_ANNEAL_EXP:
                    c = (int64_t)std::floor(k0 * std::exp(-t / param) + 1e-9); break;
                case ST3_ANNEAL_DROP:
                    c = (int64_t)k0 - (int64_t)param * t; break;
                default:
                    c = k0;
            }
            if (c < 0) c = 0;
            if (c > k0) c = k0;
            keep_lt[(int64_t)l * (T + 1) + t] = (int32_t)c;
        }
    }
    return ST3_OK;
}

extern "C" int64_t st3_kv_bytes(int32_t batch, int32_t heads, int32_t head_dim, int32_t dtype,
                                const int32_t* kv_lens, int32_t L) {
    if (!kv_lens || batch < 0 || heads < 0 || head_dim < 0 || L < 0) return -1;
    int64_t rows = 0;
    for (int32_t l = 0; l < L; ++l) rows += kv_lens[l];
    return (int64_t)batch * rows * 2 * heads * head_dim * st3::elem_bytes(dtype);
}
