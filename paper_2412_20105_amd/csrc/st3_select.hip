// Top-k selection of visual tokens by attention mass (Eq. 3), the in-place compaction of rows
// that follows it (Alg. 1/3: V = V[T]), and the per-layer, per-step eviction of visual KV rows
// (Eq. 7, Alg. 3 VTA branch).
//
// Selection is an exact radix select on the order-preserving 32-bit image of the float32 score
// (4 passes of 8 bits, histogram in LDS), followed - only when the k-th score is shared - by a
// second radix select on the tie ids, so that the result is the unique top-k set under the total
// order (score descending, id ascending).  One workgroup per sequence.
#include "st3_evict.h"

namespace st3 {

namespace {


// ---------------------------------------------------------------------------------------------
// st3_select_topk
// ---------------------------------------------------------------------------------------------
struct TopkArgs {
    const float* scores;
    int64_t score_stride;
    const int32_t* ids;
    int64_t id_stride;
    const int32_t* n_dev;
    int32_t n, k;
    uint8_t* mask;
    int32_t* idx;
    int64_t idx_stride;
};

__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(TopkArgs a) {
    __shared__ SelShared sm;
    const int b = blockIdx.x, tid = threadIdx.x;
    int n = a.n_dev ? a.n_dev[b] : a.n;
    n = max(0, min(n, a.n));
    const int k = min(a.k, n);
    const float* scores = a.scores + b * a.score_stride;
    const int32_t* ids = a.ids ? a.ids + b * a.id_stride : nullptr;
    uint8_t* mask = a.mask ? a.mask + (int64_t)b * a.n : nullptr;
    int32_t* idx = a.idx ? a.idx + (int64_t)b * a.idx_stride : nullptr;
    const bool staged = n <= kSelLdsKeys;
    uint32_t thr = 0, thr_id = 0;
    bool all_ties = true;
    if (k > 0 && k < n) mark_topk(scores, ids, n, k, staged, sm, thr, thr_id, all_ties);
    int base = 0;
    const int n_pad = (a.n + kSelThreads - 1) / kSelThreads * kSelThreads;
    for (int p0 = 0; p0 < n_pad; p0 += kSelThreads) {
        const int p = p0 + tid;
        bool keep = false;
        if (p < n) {
            if (k >= n) keep = true;
            else if (k > 0) {
                uint32_t key = staged ? sm.keys[p] : score_key(scores[p]);
                uint32_t idkey = ~(uint32_t)(ids ? ids[p] : p);
                keep = is_kept(key, idkey, thr, thr_id, all_ties);
            }
        }
        if (mask && p < a.n) mask[p] = keep ? 1 : 0;
        int incl = block_incl_scan(keep ? 1 : 0, sm);
        if (keep && idx && base + incl - 1 < a.k) idx[base + incl - 1] = p;
        __syncthreads();
        if (tid == kSelThreads - 1) sm.red = incl;
        __syncthreads();
        base += sm.red;
    }
    if (idx) for (int i = k + tid; i < a.k; i += kSelThreads) idx[i] = -1;
}

// ---------------------------------------------------------------------------------------------
// st3_compact_rows: stable in-place gather.  grid (slabs, inner, batch).
// Destination rows are produced in ascending chunks; a chunk is loaded completely before any of
// it is stored, and since keep_idx is ascending with keep_idx[r] >= r no later chunk reads a row
// an earlier chunk has overwritten.
// ---------------------------------------------------------------------------------------------
struct CompactArgs {
    char* rows;
    int64_t stride_b, stride_inner, stride_row;     // bytes
    int32_t row_units, slab_units, unit_bytes;      // a unit is 16 or 4 bytes
    const int32_t* idx;
    int64_t idx_stride;
    int32_t k, n, tail;
};

template <typename V>
__global__ __launch_bounds__(256) void compact_rows_kernel(CompactArgs a) {
    constexpr int UR = 4;
    __shared__ int sm_kb;
    __shared__ int sm_cnt[4];
    const int tid = threadIdx.x, b = blockIdx.z;
    const int32_t* idx = a.idx + (int64_t)b * a.idx_stride;
    // length of the leading run of valid indices (0 <= idx < n): position of the first invalid entry
    int local = a.k;
    for (int i = tid; i < a.k; i += 256)
        if (idx[i] < 0 || idx[i] >= a.n) { local = i; break; }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) local = min(local, __shfl_xor(local, off));
    if (tid % kWave == 0) sm_cnt[tid / kWave] = local;
    __syncthreads();
    if (tid == 0) sm_kb = min(min(sm_cnt[0], sm_cnt[1]), min(sm_cnt[2], sm_cnt[3]));
    __syncthreads();
    const int kb = sm_kb;
    const int total = kb + a.tail;
    char* strip = a.rows + b * a.stride_b + (int64_t)blockIdx.y * a.stride_inner;
    const int rows_per_pass = 256 / a.slab_units;
    const int rr = tid / a.slab_units;
    const int cu = blockIdx.x * a.slab_units + tid % a.slab_units;
    const bool col_ok = cu < a.row_units;
    for (int r0 = 0; r0 < total; r0 += UR * rows_per_pass) {
        V tmp[UR];
        int dst[UR];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            int r = r0 + u * rows_per_pass + rr;
            dst[u] = -1;
            if (r < total && col_ok) {
                int src = r < kb ? idx[r] : a.n + (r - kb);
                if (src > r && src < a.n + a.tail) {     // src == r: already in place
                    tmp[u] = *reinterpret_cast<const V*>(strip + src * a.stride_row + (int64_t)cu * sizeof(V));
                    dst[u] = r;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < UR; ++u)
            if (dst[u] >= 0) *reinterpret_cast<V*>(strip + dst[u] * a.stride_row + (int64_t)cu * sizeof(V)) = tmp[u];
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// Decode-time eviction: ranking + move list + column update (one workgroup per sequence), then
// a second kernel that applies the move list to every (b,h) strip of K and V.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void evict_plan_kernel(EvictArgs a) {
    __shared__ SelShared sm;
    evict_plan_body(a, blockIdx.x, sm);
}

// ---- st3_gather_rows: out-of-place gather of kept rows, several tensors per launch -------------
struct GatherArgs {
    st3_gather_pair pair[ST3_MAX_GATHER];
    const int32_t* idx;
    int64_t idx_stride;
    int32_t n_pairs, vecs_per_row, vpr_shift, head, k, n, tail;     // vpr_shift >= 0: vecs_per_row == 1 << vpr_shift
};

// grid (ceil(rows*vecs_per_row / (256*UR)), inner, batch*n_pairs); a thread moves UR 16-byte vectors.
#ifndef ST3_GATHER_UR
#define ST3_GATHER_UR 4         // 8 was measured 2x slower, 1-4 alike
#endif
#ifndef ST3_GATHER_NT
#define ST3_GATHER_NT 1
#endif
constexpr int kGatherUR = ST3_GATHER_UR;
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherArgs a) {
    constexpr int UR = kGatherUR;
    const int p = blockIdx.z % a.n_pairs, b = blockIdx.z / a.n_pairs;
    const st3_gather_pair& pr = a.pair[p];
    const char* src = reinterpret_cast<const char*>(pr.src) + b * pr.src_stride_b + (int64_t)blockIdx.y * pr.src_stride_inner;
    char* dst = reinterpret_cast<char*>(pr.dst) + b * pr.dst_stride_b + (int64_t)blockIdx.y * pr.dst_stride_inner;
    const int32_t* idx = a.idx ? a.idx + (int64_t)b * a.idx_stride : nullptr;
    const int rows = a.head + a.k + a.tail;
    const uint32_t total = (uint32_t)rows * (uint32_t)a.vecs_per_row;      // < 2^31, checked on the host
    const uint32_t base = blockIdx.x * (256u * UR) + threadIdx.x;
    u32x4_v tmp[UR];
    int64_t doff[UR];
#pragma unroll
    for (int u = 0; u < UR; ++u) {
        const uint32_t e = base + (uint32_t)u * 256u;
        doff[u] = -1;
        if (e < total) {
            // 32-bit index arithmetic, a shift when the row is a power of two vectors long: a 64-bit
            // division per 16 bytes moved made this kernel ALU bound
            const int r = a.vpr_shift >= 0 ? (int)(e >> a.vpr_shift) : (int)(e / (uint32_t)a.vecs_per_row);
            const int vec = (int)(e - (uint32_t)r * (uint32_t)a.vecs_per_row);
            int sr;
            if (r < a.head) sr = r;
            else if (r < a.head + a.k) {
                const int j = idx ? idx[r - a.head] : r - a.head;
                sr = (j >= 0 && j < a.n) ? a.head + j : -1;
            } else sr = r - a.k + a.n;
            if (sr >= 0) {
#if ST3_GATHER_NT
                tmp[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_v*>(src + sr * pr.src_stride_row + (int64_t)vec * 16));
#else
                tmp[u] = *reinterpret_cast<const u32x4_v*>(src + sr * pr.src_stride_row + (int64_t)vec * 16);
#endif
                doff[u] = r * pr.dst_stride_row + (int64_t)vec * 16;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < UR; ++u)
        if (doff[u] >= 0) *reinterpret_cast<u32x4_v*>(dst + doff[u]) = tmp[u];
}

struct ApplyArgs {
    char* k;
    char* v;
    int64_t stride_b, stride_h, stride_t;   // bytes
    const int32_t* move_cnt;
    const int32_t* moves;
    int32_t max_moves, H, vecs_per_row;
    int32_t vecs_per_part;      // 16-byte vectors of a row that one workgroup moves (vecs_per_row / gridDim.z)
};

// grid (2*H, B, parts): x < H moves K rows of head x, x >= H moves V rows of head x-H; z picks the
// columns [z * vecs_per_part, (z+1) * vecs_per_part) of every row.  The parts of a strip share
// nothing - each applies the whole list, in order, to its own columns - so when the strips are few
// each is moved by two workgroups, half a row per workgroup.
// Moves are applied in list order in chunks; a chunk is loaded completely before it is stored.
// The plan kernel orders the list so that no move reads a row that an earlier chunk has written
// unless that is the intended (already shifted) content.
#ifndef ST3_APPLY_UR
#define ST3_APPLY_UR 16     // 4 -> 16: 4.1 -> 4.8 TB/s read+write (plan launch included) for a stable eviction of 288 rows
#endif
__global__ __launch_bounds__(256) void evict_apply_kernel(ApplyArgs a) {
    constexpr int UR = ST3_APPLY_UR;        // 16-byte loads in flight per thread: a chunk is UR * 256 * 16 bytes
    const int b = blockIdx.y, tid = threadIdx.x;
    const int M = min(a.move_cnt[b], a.max_moves);
    if (M <= 0) return;
    if ((int)blockIdx.x < a.H && a.k == nullptr) return;    // a layer that caches V only
    const int h = blockIdx.x % a.H;
    char* strip = (blockIdx.x < a.H ? a.k : a.v) + b * a.stride_b + h * a.stride_h;
    const int32_t* mv = a.moves + (int64_t)b * a.max_moves * 2;
    const int rpp = 256 / a.vecs_per_part;
    const int rr = tid / a.vecs_per_part;
    const int64_t cb = (int64_t)((int)blockIdx.z * a.vecs_per_part + tid % a.vecs_per_part) * 16;
    for (int c0 = 0; c0 < M; c0 += UR * rpp) {
        u32x4_v tmp[UR];
        int dst[UR];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            int i = c0 + u * rpp + rr;
            dst[u] = -1;
            if (i < M) {
                dst[u] = mv[2 * i];
                // every row is read once and written once: keep it out of the way of the caches' other tenants
                tmp[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_v*>(strip + mv[2 * i + 1] * a.stride_t + cb));
            }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < UR; ++u)
            if (dst[u] >= 0) *reinterpret_cast<u32x4_v*>(strip + dst[u] * a.stride_t + cb) = tmp[u];
        __syncthreads();
    }
}

}  // namespace

st3_status validate_kv(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg);
st3_status validate_kv_value_only(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg);

// Rows are moved inside the plan kernel when the mode is HOLE_FILL and few rows can be evicted per
// sequence; larger evictions and STABLE mode go through evict_apply_kernel, which has a workgroup
// per strip but is a launch of its own per layer.  A plan workgroup moves a row on all 2*H strips in
// about 2 us (measured, H = 40, bf16 d = 128), a plan + apply pair costs about 10 us more than a plan
// alone: so up to 48 evicted rows stay in the plan when the plans of many layers share a launch
// (the apply launches they save are per layer), and only a handful when a layer is planned alone
// (each evicted row is one move with a fixed tail, two without).
constexpr int kInlineEvictBatched = 48;
constexpr int kInlineEvictAloneFixedTail = 8;
constexpr int kInlineEvictAlone = 4;

st3_status build_evict_args(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                            float* score_col, int32_t* id_col, int64_t col_stride, int32_t keep_count, int32_t mode,
                            void* workspace, size_t workspace_bytes, int appended, float* mass_dst,
                            int64_t mass_stride, EvictArgs& ea, bool& needs_apply, bool batched,
                            const void* mass_workspace, int32_t mass_capacity) {
    const int B = shape->batch, H = shape->heads, D = shape->head_dim;
    if (seg->max_vis_len > kSelLdsKeys) return ST3_ERR_UNSUPPORTED;
    const DecodeWs wl = decode_ws(B, H, D, kv->capacity);
    if (workspace_bytes < wl.total) return ST3_ERR_WORKSPACE_TOO_SMALL;
    char* ws = reinterpret_cast<char*>(workspace);
    const int eb = kv_elem_bytes(shape, kv);
    const bool evicting = keep_count >= 0 && keep_count < seg->max_vis_len;
    ea = EvictArgs{};
    ea.score_col = score_col; ea.id_col = id_col; ea.col_stride = col_stride;
    ea.vis_len = seg->vis_len; ea.kv_len = seg->kv_len; ea.tail_start = seg->tail_start;
    ea.sys_len = seg->sys_len; ea.max_vis = seg->max_vis_len; ea.max_kv = seg->max_kv_len;
    ea.keep_count = evicting ? keep_count : -1; ea.mode = mode;
    ea.move_cnt = reinterpret_cast<int32_t*>(ws + wl.moves_cnt);
    ea.moves = reinterpret_cast<int32_t*>(ws + wl.moves);
    ea.max_moves = wl.max_moves;
    ea.appended = appended; ea.capacity = kv->capacity;
    const int inline_limit = batched ? kInlineEvictBatched
                                     : (seg->tail_start != nullptr ? kInlineEvictAloneFixedTail : kInlineEvictAlone);
    ea.inline_apply = evicting && mode == ST3_HOLE_FILL && (seg->max_vis_len - keep_count) <= inline_limit;
    ea.k = reinterpret_cast<char*>(kv->k); ea.v = reinterpret_cast<char*>(kv->v);
    ea.stride_b = kv->stride_b * eb; ea.stride_h = kv->stride_h * eb; ea.stride_t = kv->stride_t * eb;
    ea.H = H; ea.vecs_per_row = D * eb / 16;
    if (mass_dst != nullptr) {
        const char* mws = mass_workspace ? reinterpret_cast<const char*>(mass_workspace) : ws;
        const DecodeWs ml = mass_workspace ? decode_ws(B, H, D, mass_capacity) : wl;
        ea.part_ml = reinterpret_cast<const float*>(mws + ml.part_ml);
        ea.logits = reinterpret_cast<const float*>(mws + ml.logits);
        ea.pending = reinterpret_cast<const int32_t*>(mws + ml.pending);
        ea.nsplit_cap = ml.nsplit_cap;
        if (mass_workspace) ea.capacity = mass_capacity;
        ea.mass_dst = mass_dst; ea.mass_stride = mass_stride;
    }
    needs_apply = evicting && !ea.inline_apply;
    return ST3_OK;
}

void launch_evict_plan(const EvictArgs& ea, int B, hipStream_t st) {
    evict_plan_kernel<<<B, kSelThreads, 0, st>>>(ea);
}

// Up to kPlanBatch plans travel by value in the kernel arguments; grid (B, layers of the batch).
struct EvictBatch {
    EvictArgs layer[kPlanBatch];
};
static_assert(sizeof(EvictBatch) <= 4000, "plans of one batch must fit the kernel argument segment");

constexpr int kMergeHeads = 8;      // heads whose chunk partials one merge workgroup combines

// grid (B, layers of the batch, 1 + merge workgroups): z = 0 runs the plan of (sequence x, layer y);
// z >= 1 merges the chunk partials of that layer's attention output for kMergeHeads heads (only
// launched when some layer of the batch left partials to merge).
__global__ __launch_bounds__(kSelThreads) void evict_plan_batch_kernel(EvictBatch batch) {
    __shared__ SelShared sm;
    const EvictArgs& a = batch.layer[blockIdx.y];
    if (blockIdx.z == 0) {
        evict_plan_body(a, blockIdx.x, sm);
    } else if (a.merge_out != nullptr && a.pending != nullptr) {
        const int h0 = ((int)blockIdx.z - 1) * kMergeHeads;
        if (h0 < a.H) merge_chunks(a, blockIdx.x, h0, h0 + kMergeHeads);
    }
}

void launch_evict_plan_batch(const EvictArgs* plans, int n, int B, hipStream_t st) {
    for (int i0 = 0; i0 < n; i0 += kPlanBatch) {
        const int cnt = n - i0 < kPlanBatch ? n - i0 : kPlanBatch;
        EvictBatch batch;
        int merge_heads = 0;
        for (int i = 0; i < cnt; ++i) {
            batch.layer[i] = plans[i0 + i];
            if (plans[i0 + i].merge_out != nullptr && plans[i0 + i].H > merge_heads) merge_heads = plans[i0 + i].H;
        }
        for (int i = cnt; i < kPlanBatch; ++i) batch.layer[i] = EvictArgs{};
        const int merge_wgs = (merge_heads + kMergeHeads - 1) / kMergeHeads;
        evict_plan_batch_kernel<<<dim3(B, cnt, 1 + merge_wgs), kSelThreads, 0, st>>>(batch);
    }
}

// The same with the plans read from device memory, where the layers' attention launches left them
// (PlanStash): up to kPlanTableMax layers per launch.  grid as above.
struct PlanTable {
    const EvictArgs* layer[kPlanTableMax];
};

__global__ __launch_bounds__(kSelThreads) void evict_plan_table_kernel(PlanTable table) {
    __shared__ SelShared sm;
    // read once, ahead of every store of this kernel: uniform address, so the fields arrive in scalar registers
    const EvictArgs a = *table.layer[blockIdx.y];
    if (blockIdx.z == 0) {
        evict_plan_body(a, blockIdx.x, sm);
    } else if (a.merge_out != nullptr && a.pending != nullptr) {
        const int h0 = ((int)blockIdx.z - 1) * kMergeHeads;
        if (h0 < a.H) merge_chunks(a, blockIdx.x, h0, h0 + kMergeHeads);
    }
}

void launch_evict_plan_table(const EvictArgs* const* stashed, const EvictArgs* plans, int n, int B, hipStream_t st) {
    for (int i0 = 0; i0 < n; i0 += kPlanTableMax) {
        const int cnt = n - i0 < kPlanTableMax ? n - i0 : kPlanTableMax;
        PlanTable table;
        int merge_heads = 0;
        for (int i = 0; i < cnt; ++i) {
            table.layer[i] = stashed[i0 + i];
            if (plans[i0 + i].merge_out != nullptr && plans[i0 + i].H > merge_heads) merge_heads = plans[i0 + i].H;
        }
        for (int i = cnt; i < kPlanTableMax; ++i) table.layer[i] = nullptr;
        const int merge_wgs = (merge_heads + kMergeHeads - 1) / kMergeHeads;
        evict_plan_table_kernel<<<dim3(B, cnt, 1 + merge_wgs), kSelThreads, 0, st>>>(table);
    }
}

void launch_evict_apply(const EvictArgs& ea, int B, hipStream_t st) {
    ApplyArgs aa{};
    aa.k = ea.k; aa.v = ea.v;
    aa.stride_b = ea.stride_b; aa.stride_h = ea.stride_h; aa.stride_t = ea.stride_t;
    aa.move_cnt = ea.move_cnt; aa.moves = ea.moves; aa.max_moves = ea.max_moves; aa.H = ea.H;
    aa.vecs_per_row = ea.vecs_per_row;
    // two column halves per strip while the strips are few and a half is whole 128-byte lines: measured read+write rate of a
    // stable eviction, one part -> two, 512 strips (high-resolution shape, batch 8) 3.0 -> 3.9 TB/s, 640 strips (13B shape,
    // batch 8) 3.0 -> 3.8, 1280 strips (batch 16) 4.8 -> 4.7
    const int parts = (2 * ea.H * B <= 1024 && ea.vecs_per_row % 16 == 0) ? 2 : 1;
    aa.vecs_per_part = ea.vecs_per_row / parts;
    evict_apply_kernel<<<dim3(2 * ea.H, B, parts), 256, 0, st>>>(aa);
}


// Eviction plan (+ optional append bookkeeping, finishing of the mass and in-kernel row moves),
// then the separate move kernel when the plan kernel does not move the rows itself.
//   appended:   the attention kernel has just written one row beyond kv_len[b]; it is counted here
//   mass_dst:   where the mass of the attention launch before this call is finished (null: skip)
st3_status enqueue_select_compact(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                                  float* score_col, int32_t* id_col, int64_t col_stride, int32_t keep_count,
                                  int32_t mode, void* workspace, size_t workspace_bytes, hipStream_t st,
                                  int appended, float* mass_dst, int64_t mass_stride) {
    EvictArgs ea;
    bool needs_apply = false;
    st3_status s = build_evict_args(shape, kv, seg, score_col, id_col, col_stride, keep_count, mode, workspace,
                                    workspace_bytes, appended, mass_dst, mass_stride, ea, needs_apply, false);
    if (s != ST3_OK) return s;
    launch_evict_plan(ea, shape->batch, st);
    if (needs_apply) launch_evict_apply(ea, shape->batch, st);
    return check_launch();
}

// ---------------------------------------------------------------------------------------------
// Diagnostics on mass vectors: Overlap_n (Eq. 10) and cosine similarity (Eq. 4-5).
// ---------------------------------------------------------------------------------------------
namespace {

constexpr int kDiagIdSpace = 16384;

struct OverlapArgs {
    const float* score_a; const int32_t* ids_a; int64_t stride_a; const int32_t* n_a_dev; int32_t n_a;
    const float* score_b; const int32_t* ids_b; int64_t stride_b; const int32_t* n_b_dev; int32_t n_b;
    int32_t k, id_space;
    int32_t* overlap;       // [B] |TopK(a) ^ TopK(b)|
    int32_t* topk_a;        // [B] |TopK(a)| = min(k, n_a[b])
};

// One workgroup per sequence.  TopK(a) is marked in an LDS bitmap indexed by token id; the
// members of TopK(b) whose id is marked are counted.
__global__ __launch_bounds__(kSelThreads) void overlap_topk_kernel(OverlapArgs a) {
    __shared__ SelShared sm;
    __shared__ uint32_t seen[kDiagIdSpace / 32];
    __shared__ int sm_count;
    const int b = blockIdx.x, tid = threadIdx.x;
    for (int i = tid; i < kDiagIdSpace / 32; i += kSelThreads) seen[i] = 0u;
    if (tid == 0) sm_count = 0;
    __syncthreads();
    for (int side = 0; side < 2; ++side) {
        const float* scores = (side ? a.score_b + b * a.stride_b : a.score_a + b * a.stride_a);
        const int32_t* ids = (side ? a.ids_b + b * a.stride_b : a.ids_a + b * a.stride_a);
        const int32_t* n_dev = side ? a.n_b_dev : a.n_a_dev;
        int n = n_dev ? n_dev[b] : (side ? a.n_b : a.n_a);
        n = max(0, min(n, side ? a.n_b : a.n_a));
        const int k = min(a.k, n);
        uint32_t thr = 0, thr_id = 0;
        bool all_ties = true;
        if (k > 0 && k < n) mark_topk(scores, ids, n, k, true, sm, thr, thr_id, all_ties);
        else __syncthreads();
        int local = 0;
        for (int p = tid; p < n; p += kSelThreads) {
            bool keep = k >= n;
            if (!keep && k > 0) keep = is_kept(sm.keys[p], ~(uint32_t)ids[p], thr, thr_id, all_ties);
            const int id = ids[p];
            if (!keep || id < 0 || id >= a.id_space) continue;
            if (side == 0) atomicOr(&seen[id >> 5], 1u << (id & 31));
            else local += (seen[id >> 5] >> (id & 31)) & 1u;
        }
        if (side == 0 && tid == 0) a.topk_a[b] = k;
        if (side == 1 && local) atomicAdd(&sm_count, local);
        __syncthreads();
    }
    if (tid == 0) a.overlap[b] = sm_count;
}

struct CosineArgs {
    const float* va; const int32_t* ids_a; int64_t stride_a; const int32_t* n_a_dev; int32_t n_a;
    const float* vb; const int32_t* ids_b; int64_t stride_b; const int32_t* n_b_dev; int32_t n_b;
    int32_t id_space;
    float* cosine;          // [B]
};

__device__ __forceinline__ float block_sum(float v, float* sm4) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if (threadIdx.x % kWave == 0) sm4[threadIdx.x / kWave] = v;
    __syncthreads();
    return (sm4[0] + sm4[1]) + (sm4[2] + sm4[3]);
}

// One workgroup per sequence.  Entries are matched by token id (ids_x == null: by position);
// tokens present on one side only count as zero on the other.  fp32 sums in a fixed order.
__global__ __launch_bounds__(kSelThreads) void cosine_kernel(CosineArgs a) {
    __shared__ int16_t pos_b[kDiagIdSpace];
    __shared__ float sm4[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    const float* va = a.va + b * a.stride_a;
    const float* vb = a.vb + b * a.stride_b;
    const int32_t* ia = a.ids_a ? a.ids_a + b * a.stride_a : nullptr;
    const int32_t* ib = a.ids_b ? a.ids_b + b * a.stride_b : nullptr;
    const int na = max(0, min(a.n_a_dev ? a.n_a_dev[b] : a.n_a, a.n_a));
    const int nb = max(0, min(a.n_b_dev ? a.n_b_dev[b] : a.n_b, a.n_b));
    for (int i = tid; i < a.id_space; i += kSelThreads) pos_b[i] = -1;
    __syncthreads();
    float sbb = 0.f;
    for (int p = tid; p < nb; p += kSelThreads) {
        const int id = ib ? ib[p] : p;
        if (id >= 0 && id < a.id_space) pos_b[id] = (int16_t)p;
        sbb = fmaf(vb[p], vb[p], sbb);
    }
    __syncthreads();
    float saa = 0.f, sab = 0.f;
    for (int p = tid; p < na; p += kSelThreads) {
        const int id = ia ? ia[p] : p;
        const float x = va[p];
        saa = fmaf(x, x, saa);
        if (id >= 0 && id < a.id_space && pos_b[id] >= 0) sab = fmaf(x, vb[pos_b[id]], sab);
    }
    const float taa = block_sum(saa, sm4), tbb = block_sum(sbb, sm4), tab = block_sum(sab, sm4);
    if (tid == 0) a.cosine[b] = (taa > 0.f && tbb > 0.f) ? tab / (sqrtf(taa) * sqrtf(tbb)) : 0.f;
}

}  // namespace

}  // namespace st3

extern "C" st3_status st3_overlap_topk(const float* score_a, const int32_t* ids_a, int64_t stride_a,
                                       const int32_t* n_a_dev, int32_t n_a, const float* score_b,
                                       const int32_t* ids_b, int64_t stride_b, const int32_t* n_b_dev, int32_t n_b,
                                       int32_t batch, int32_t k, int32_t id_space, int32_t* overlap, int32_t* topk_a,
                                       void* stream) {
    if (!score_a || !ids_a || !score_b || !ids_b || !overlap || !topk_a) return ST3_ERR_INVALID_ARG;
    if (batch <= 0 || n_a < 0 || n_b < 0 || k < 0 || stride_a < n_a || stride_b < n_b) return ST3_ERR_INVALID_ARG;
    if (n_a > st3::kSelLdsKeys || n_b > st3::kSelLdsKeys || id_space <= 0 || id_space > st3::kDiagIdSpace)
        return ST3_ERR_UNSUPPORTED;
    st3::OverlapArgs a{score_a, ids_a, stride_a, n_a_dev, n_a, score_b, ids_b, stride_b, n_b_dev, n_b, k, id_space,
                       overlap, topk_a};
    st3::overlap_topk_kernel<<<batch, st3::kSelThreads, 0, reinterpret_cast<hipStream_t>(stream)>>>(a);
    return st3::check_launch();
}

extern "C" st3_status st3_cosine_similarity(const float* va, const int32_t* ids_a, int64_t stride_a,
                                            const int32_t* n_a_dev, int32_t n_a, const float* vb,
                                            const int32_t* ids_b, int64_t stride_b, const int32_t* n_b_dev,
                                            int32_t n_b, int32_t batch, int32_t id_space, float* cosine, void* stream) {
    if (!va || !vb || !cosine) return ST3_ERR_INVALID_ARG;
    if (batch <= 0 || n_a < 0 || n_b < 0 || stride_a < n_a || stride_b < n_b) return ST3_ERR_INVALID_ARG;
    if (id_space <= 0 || id_space > st3::kDiagIdSpace || n_a > 32767 || n_b > 32767) return ST3_ERR_UNSUPPORTED;
    st3::CosineArgs a{va, ids_a, stride_a, n_a_dev, n_a, vb, ids_b, stride_b, n_b_dev, n_b, id_space, cosine};
    st3::cosine_kernel<<<batch, st3::kSelThreads, 0, reinterpret_cast<hipStream_t>(stream)>>>(a);
    return st3::check_launch();
}

extern "C" st3_status st3_select_topk(const float* scores, int64_t score_stride, const int32_t* tie_ids,
                                      int64_t id_stride, int32_t batch, const int32_t* n_dev, int32_t n, int32_t k,
                                      uint8_t* keep_mask, int32_t* keep_idx, int64_t idx_stride, void* stream) {
    if (!scores || batch <= 0 || n < 0 || k < 0 || k > n) return ST3_ERR_INVALID_ARG;
    if (keep_idx && idx_stride < k) return ST3_ERR_INVALID_ARG;
    if (n > 16384 || batch > 65535 * 32) return ST3_ERR_UNSUPPORTED;
    if (score_stride < n || (tie_ids && id_stride < n)) return ST3_ERR_INVALID_ARG;
    if (n == 0) return ST3_OK;
    st3::TopkArgs a{};
    a.scores = scores; a.score_stride = score_stride; a.ids = tie_ids; a.id_stride = id_stride;
    a.n_dev = n_dev; a.n = n; a.k = k; a.mask = keep_mask; a.idx = keep_idx; a.idx_stride = idx_stride;
    st3::select_topk_kernel<<<batch, st3::kSelThreads, 0, reinterpret_cast<hipStream_t>(stream)>>>(a);
    return st3::check_launch();
}

extern "C" st3_status st3_compact_rows(void* rows, int32_t batch, int32_t inner, int64_t stride_b_bytes,
                                       int64_t stride_inner_bytes, int64_t stride_row_bytes, int32_t row_bytes,
                                       const int32_t* keep_idx, int64_t idx_stride, int32_t k, int32_t n,
                                       int32_t tail_rows, void* stream) {
    if (!rows || !keep_idx || batch <= 0 || inner <= 0 || k < 0 || n < 0 || k > n || tail_rows < 0)
        return ST3_ERR_INVALID_ARG;
    if (idx_stride < k) return ST3_ERR_INVALID_ARG;
    if (row_bytes <= 0 || row_bytes % 4 || stride_row_bytes < row_bytes) return ST3_ERR_INVALID_ARG;
    if (batch > 65535 || inner > 65535) return ST3_ERR_UNSUPPORTED;
    if (k + tail_rows == 0) return ST3_OK;
    const bool vec16 = (row_bytes % 16 == 0) && (stride_row_bytes % 16 == 0) && (stride_b_bytes % 16 == 0) &&
                       (stride_inner_bytes % 16 == 0) && st3::aligned16(rows);
    if (!vec16 && ((stride_row_bytes % 4) || (stride_b_bytes % 4) || (stride_inner_bytes % 4) ||
                   (reinterpret_cast<uintptr_t>(rows) & 3)))
        return ST3_ERR_INVALID_ARG;
    st3::CompactArgs a{};
    a.rows = reinterpret_cast<char*>(rows);
    a.stride_b = stride_b_bytes; a.stride_inner = stride_inner_bytes; a.stride_row = stride_row_bytes;
    a.unit_bytes = vec16 ? 16 : 4;
    a.row_units = row_bytes / a.unit_bytes;
    int slab = 1;
    while (slab * 2 <= a.row_units && slab * 2 <= 256) slab *= 2;
    a.slab_units = slab;
    a.idx = keep_idx; a.idx_stride = idx_stride; a.k = k; a.n = n; a.tail = tail_rows;
    dim3 grid((a.row_units + slab - 1) / slab, inner, batch);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (vec16) st3::compact_rows_kernel<uint4><<<grid, 256, 0, st>>>(a);
    else st3::compact_rows_kernel<uint32_t><<<grid, 256, 0, st>>>(a);
    return st3::check_launch();
}

extern "C" st3_status st3_gather_rows(const st3_gather_pair* pairs, int32_t n_pairs, int32_t batch, int32_t inner,
                                      int32_t row_bytes, int32_t head_rows, const int32_t* keep_idx, int64_t idx_stride,
                                      int32_t k, int32_t n, int32_t tail_rows, void* stream) {
    using namespace st3;
    if (!pairs || n_pairs <= 0 || n_pairs > ST3_MAX_GATHER || batch <= 0 || inner <= 0) return ST3_ERR_INVALID_ARG;
    if (row_bytes <= 0 || row_bytes % 16 || head_rows < 0 || k < 0 || n < 0 || k > n || tail_rows < 0)
        return ST3_ERR_INVALID_ARG;
    if (!keep_idx && k != n) return ST3_ERR_INVALID_ARG;
    if (keep_idx && idx_stride < k) return ST3_ERR_INVALID_ARG;
    if ((int64_t)batch * n_pairs > 65535 || inner > 65535) return ST3_ERR_UNSUPPORTED;
    const int64_t src_rows = (int64_t)head_rows + n + tail_rows, dst_rows = (int64_t)head_rows + k + tail_rows;
    GatherArgs a{};
    for (int p = 0; p < n_pairs; ++p) {
        const st3_gather_pair& g = pairs[p];
        if (!g.src || !g.dst || !aligned16(g.src) || !aligned16(g.dst)) return ST3_ERR_INVALID_ARG;
        const int64_t st[6] = {g.src_stride_b, g.src_stride_inner, g.src_stride_row,
                               g.dst_stride_b, g.dst_stride_inner, g.dst_stride_row};
        for (int64_t v : st) if (v < 0 || v % 16) return ST3_ERR_INVALID_ARG;
        if (g.src_stride_row < row_bytes || g.dst_stride_row < row_bytes) return ST3_ERR_INVALID_ARG;
        // the whole source and destination regions of this pair must be disjoint
        const char* s0 = reinterpret_cast<const char*>(g.src);
        const char* d0 = reinterpret_cast<const char*>(g.dst);
        const int64_t s_ext = (batch - 1) * g.src_stride_b + (inner - 1) * g.src_stride_inner +
                              (src_rows > 0 ? (src_rows - 1) * g.src_stride_row + row_bytes : 0);
        const int64_t d_ext = (batch - 1) * g.dst_stride_b + (inner - 1) * g.dst_stride_inner +
                              (dst_rows > 0 ? (dst_rows - 1) * g.dst_stride_row + row_bytes : 0);
        if (s0 < d0 + d_ext && d0 < s0 + s_ext) return ST3_ERR_INVALID_ARG;
        a.pair[p] = g;
    }
    if (dst_rows == 0) return ST3_OK;
    a.idx = keep_idx; a.idx_stride = idx_stride; a.n_pairs = n_pairs; a.vecs_per_row = row_bytes / 16;
    a.head = head_rows; a.k = k; a.n = n; a.tail = tail_rows;
    const int64_t total = dst_rows * a.vecs_per_row;
    if (total >= 0x7fffffff) return ST3_ERR_UNSUPPORTED;           // the kernel indexes a strip with 32 bits
    a.vpr_shift = -1;
    for (int sh = 0; sh < 31; ++sh)
        if ((1 << sh) == a.vecs_per_row) a.vpr_shift = sh;
    const int64_t blocks = (total + 256 * kGatherUR - 1) / (256 * kGatherUR);
    gather_rows_kernel<<<dim3((unsigned)blocks, inner, batch * n_pairs), 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(a);
    return check_launch();
}

extern "C" st3_status st3_select_compact_layer(const st3_attn_shape* shape, const st3_kv_layer* kv,
                                               const st3_segments* seg, float* score_col, int32_t* id_col,
                                               int64_t col_stride, int32_t keep_count, int32_t mode,
                                               void* workspace, size_t workspace_bytes, void* stream) {
    st3_status s = st3::check_shape(shape);
    if (s != ST3_OK) return s;
    s = (kv && !kv->k) ? st3::validate_kv_value_only(shape, kv, seg) : st3::validate_kv(shape, kv, seg);
    if (s != ST3_OK) return s;
    if (!score_col || !id_col || !workspace || keep_count < 0) return ST3_ERR_INVALID_ARG;
    if (col_stride < seg->max_vis_len) return ST3_ERR_INVALID_ARG;
    if (mode != ST3_STABLE && mode != ST3_HOLE_FILL) return ST3_ERR_INVALID_ARG;
    if (!st3::aligned16(workspace)) return ST3_ERR_INVALID_ARG;
    return st3::enqueue_select_compact(shape, kv, seg, score_col, id_col, col_stride, keep_count, mode, workspace,
                                       workspace_bytes, reinterpret_cast<hipStream_t>(stream), 0, nullptr, 0);
}
