// Exact top-k selection (radix select on the order-preserving image of the fp32 score, ties by
// id) and the per-sequence eviction plan of a decode step (Eq. 3, Eq. 7, Alg. 3 VTA branch), as
// device code of the selection and eviction kernels.
#pragma once

#include "st3_decode.h"

namespace st3 {
constexpr int kSelThreads = 256;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelLdsKeys = 8192;

__device__ __forceinline__ uint32_t score_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;                       // -0.0 ranks with +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger float <-> larger key
}

struct SelShared {
    uint32_t keys[kSelLdsKeys];
    uint32_t flags[kSelLdsKeys / 32];
    int hist[256];
    int wave_tot[kSelWaves];
    int sel_bin, sel_want, sel_cnt;
    int red;
};

// Inclusive scan of one int per thread over the 256 threads of the block, in thread order.
__device__ __forceinline__ int block_incl_scan(int v, SelShared& sm) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        int t = __shfl_up(v, off);
        if (lane >= off) v += t;
    }
    __syncthreads();                                    // protects wave_tot from the previous use
    if (lane == kWave - 1) sm.wave_tot[wave] = v;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) base += (w < wave) ? sm.wave_tot[w] : 0;
    return v + base;
}

// Finds, among the elements i in [0,n) for which f(i, key) is true, the key of rank `want`
// (1-based, descending).  Returns it; `want` becomes the number of elements equal to that key
// that still belong to the top set, `ties` the number of elements equal to it.
template <class F>
__device__ __forceinline__ uint32_t radix_select_desc(F f, int n, int& want, int& ties, SelShared& sm) {
    uint32_t prefix = 0, pmask = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
        sm.hist[threadIdx.x] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < n; i += kSelThreads) {
            uint32_t key;
            if (f(i, key) && (key & pmask) == prefix) atomicAdd(&sm.hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        int v = sm.hist[255 - threadIdx.x];             // thread order = descending bin order
        int incl = block_incl_scan(v, sm);
        if (incl >= want && incl - v < want) {
            sm.sel_bin = 255 - threadIdx.x;
            sm.sel_want = want - (incl - v);
            sm.sel_cnt = v;
        }
        __syncthreads();
        prefix |= (uint32_t)sm.sel_bin << shift;
        pmask |= 255u << shift;
        want = sm.sel_want;
        ties = sm.sel_cnt;
        __syncthreads();
    }
    return prefix;
}

// Marks the top-k entries of one row in sm.flags (bit p of word p/32).  Requires n <= kSelLdsKeys
// when `staged`; otherwise keys are recomputed from global memory on every pass.
// ids == nullptr: the position is the id.
__device__ __forceinline__ void mark_topk(const float* scores, const int32_t* ids, int n, int k, bool staged, SelShared& sm,
                          uint32_t& thr, uint32_t& thr_id, bool& all_ties) {
    auto key_at = [&](int i) -> uint32_t { return staged ? sm.keys[i] : score_key(scores[i]); };
    if (staged) {
        for (int i = threadIdx.x; i < n; i += kSelThreads) sm.keys[i] = score_key(scores[i]);
        __syncthreads();
    }
    int want = k, ties = 0;
    thr = radix_select_desc([&](int i, uint32_t& key) { key = key_at(i); return true; }, n, want, ties, sm);
    all_ties = (want == ties);
    thr_id = 0;
    if (!all_ties) {
        const uint32_t t = thr;
        int want2 = want, ties2 = 0;
        thr_id = radix_select_desc(
            [&](int i, uint32_t& key) {
                key = ~(uint32_t)(ids ? ids[i] : i);    // descending on ~id == ascending on id
                return key_at(i) == t;
            },
            n, want2, ties2, sm);
    }
}

__device__ __forceinline__ bool is_kept(uint32_t key, uint32_t idkey, uint32_t thr, uint32_t thr_id, bool all_ties) {
    return key > thr || (key == thr && (all_ties || idkey >= thr_id));
}

struct EvictArgs {
    float* score_col;
    int32_t* id_col;
    int64_t col_stride;
    int32_t* vis_len;
    int32_t* kv_len;
    const int32_t* tail_start;  // [B] or null: the tail keeps its place (no tail moves, kv_len not lowered)
    int32_t sys_len, max_vis, max_kv, keep_count, mode;
    int32_t* move_cnt;          // [B]
    int32_t* moves;             // [B][max_moves][2] = (dst row, src row)
    int32_t max_moves;
    // extras used by the fused per-layer decode step
    int32_t appended;           // 1: the attention kernel has just written one more row than kv_len[b] says
    int32_t capacity;           // row stride of `logits` (capacity of the cache whose attention produced them)
    int32_t inline_apply;       // 1: HOLE_FILL moves are applied to K and V by this kernel
    char* k;
    char* v;
    int64_t stride_b, stride_h, stride_t;   // bytes
    int32_t H, vecs_per_row;
    // visual mass the attention kernel left to be finished here (all null: none)
    const float* part_ml;
    const float* logits;
    const int32_t* pending;     // [B][4] descriptor written by the attend kernel (read only: lazy layers share it)
    int32_t nsplit_cap;
    float* mass_dst;
    int64_t mass_stride;
    // chunk partials of the attention output that the attend launch left for this plan to merge
    // (whole-step call with strips cut into chunks; null: the output is complete already)
    const float* merge_part_o;  // [B,H,nsplit_cap,D]
    void* merge_out;            // [B,H,D]
    int32_t merge_D, merge_bf16;
};

__device__ __forceinline__ bool flag_at(const SelShared& sm, int p) { return (sm.flags[p >> 5] >> (p & 31)) & 1u; }

typedef uint32_t u32x4_v __attribute__((ext_vector_type(4)));

// Address of 16-byte vector `idx` of a batch of row moves: idx enumerates (move, strip, vector).
__device__ __forceinline__ char* move_addr(const EvictArgs& a, int b, const int32_t* mv, int first, int idx, int which) {
    const int strips = (a.k ? 2 : 1) * a.H;             // K may be absent (layers that keep V only)
    const int per_move = strips * a.vecs_per_row;
    const int i = first + idx / per_move;
    const int rem = idx % per_move;
    const int strip = rem / a.vecs_per_row, vec = rem % a.vecs_per_row;
    char* base = ((a.k && strip < a.H) ? a.k : a.v) + b * a.stride_b + (int64_t)(strip % a.H) * a.stride_h +
                 (int64_t)vec * 16;
    return base + mv[2 * i + which] * a.stride_t;
}

// Copies `count` rows (dst_i <- src_i, from the move list starting at entry `first`) on all
// strips of sequence b.  Callers guarantee that no destination of the batch is a source of it.
__device__ __forceinline__ void copy_rows_all_strips(const EvictArgs& a, int b, const int32_t* mv, int first, int count) {
    constexpr int UR = 16;                              // independent 16-byte loads in flight per thread
    const int total = count * (a.k ? 2 : 1) * a.H * a.vecs_per_row;
    for (int base = 0; base < total; base += UR * kSelThreads) {
        u32x4_v tmp[UR];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const int idx = base + u * kSelThreads + (int)threadIdx.x;
            if (idx < total) tmp[u] = *reinterpret_cast<const u32x4_v*>(move_addr(a, b, mv, first, idx, 1));
        }
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const int idx = base + u * kSelThreads + (int)threadIdx.x;
            if (idx < total) *reinterpret_cast<u32x4_v*>(move_addr(a, b, mv, first, idx, 0)) = tmp[u];
        }
    }
}

// Merges the chunk partials of the output rows of heads [h0, h1) of sequence b in chunk order (what
// decode_finish_kernel does when the attention is called on its own).  Runs beside the plan
// workgroup of the same sequence, which rewrites the lengths: the number of rows the attend launch
// saw therefore comes from the descriptor that launch left, not from the lengths.
__device__ __forceinline__ void merge_chunks(const EvictArgs& a, int b, int h0, int h1) {
    const int nsplit = min(a.pending[b * 4 + 1], a.nsplit_cap);
    const int chunk = max(a.pending[b * 4 + 2], 32);
    const int seen = a.pending[b * 4] >> 1;
    const int ns = seen > 0 ? min((seen + chunk - 1) / chunk, nsplit) : 0;
    if (ns <= 0) return;                                // an empty sequence had its zeros written by the attend launch
    const int D = a.merge_D;
    h1 = min(h1, a.H);
    for (int idx = threadIdx.x; idx < (h1 - h0) * D; idx += blockDim.x) {
        const int h = h0 + idx / D, d = idx % D;
        const int64_t bh = (int64_t)b * a.H + h;
        const float* ml = a.part_ml + bh * a.nsplit_cap * 2;
        float m = ml[0];
        for (int s = 1; s < ns; ++s) m = fmaxf(m, ml[2 * s]);
        float l = 0.f, o = 0.f;
        for (int s = 0; s < ns; ++s) {
            const float f = exp2_fast(ml[2 * s] - m);
            l = fmaf(ml[2 * s + 1], f, l);
            o = fmaf(a.merge_part_o[(bh * a.nsplit_cap + s) * D + d], f, o);
        }
        const float r = o / l;
        if (a.merge_bf16) reinterpret_cast<uint16_t*>(a.merge_out)[bh * D + d] = (uint16_t)f32_to_bf16_bits(r);
        else reinterpret_cast<float*>(a.merge_out)[bh * D + d] = r;
    }
}

// The whole per-sequence plan, run by one workgroup of kSelThreads threads for sequence b:
//   1. finish the visual mass the attention kernel left pending (head reduction in head order),
//   2. rank the visual rows by score_col and evict down to keep_count (columns, and - when
//      inline_apply - the K/V rows themselves),
//   3. publish the new lengths (including the row the attention kernel appended).
__device__ __forceinline__ void evict_plan_body(const EvictArgs& a, int b, SelShared& sm) {
    const int tid = threadIdx.x;
    const int n = max(0, min(a.vis_len[b], a.max_vis));
    const int len = max(0, min(a.kv_len[b] + (a.appended ? 1 : 0), a.max_kv + (a.appended ? 1 : 0)));
    const int k = a.keep_count < 0 ? n : min(a.keep_count, n);
    int new_len = len, moves_left = 0;
    if (a.pending != nullptr && a.mass_dst != nullptr) {
        // finish the mass the attention call left pending: `len` and `n` are the lengths it saw
        __shared__ float sm_hm[1024], sm_hrl[1024];
        const int valid = a.pending[b * 4] & 1;
        if (valid) {
            const int nsplit = min(a.pending[b * 4 + 1], a.nsplit_cap);
            const int chunk = max(a.pending[b * 4 + 2], 32);
            const int seen = seq_layout(a.sys_len, n, a.max_vis, len, a.tail_start, b).vlen;    // rows the attend launch saw
            const int ns = seen > 0 ? min((seen + chunk - 1) / chunk, nsplit) : 0;
            head_norms(a.part_ml, b, a.H, ns, a.nsplit_cap, sm_hm, sm_hrl);
            finish_mass(a.logits + a.sys_len, b, a.H, a.capacity, sm_hm, sm_hrl, 0, n, a.mass_dst + b * a.mass_stride);
            __syncthreads();                            // the ranking below may read these scores
        }
    }
    if (k < n && a.sys_len + n <= len) {                // something to evict, lengths consistent
        float* scores = a.score_col + b * a.col_stride;
        int32_t* ids = a.id_col + b * a.col_stride;
        int32_t* mv = a.moves + (int64_t)b * a.max_moves * 2;
        uint32_t thr = 0, thr_id = 0;
        bool all_ties = true;
        if (k > 0) mark_topk(scores, ids, n, k, true, sm, thr, thr_id, all_ties);
        // flags -> LDS bitmap (one 32-bit word per 32 positions, built from wave ballots)
        const int n_pad = (n + kSelThreads - 1) / kSelThreads * kSelThreads;
        for (int p0 = 0; p0 < n_pad; p0 += kSelThreads) {
            const int p = p0 + tid;
            bool keep = false;
            if (p < n && k > 0) keep = is_kept(sm.keys[p], ~(uint32_t)ids[p], thr, thr_id, all_ties);
            unsigned long long bal = __ballot(keep);
            if (tid % kWave == 0) {
                sm.flags[(p >> 5)] = (uint32_t)bal;
                sm.flags[(p >> 5) + 1] = (uint32_t)(bal >> 32);
            }
        }
        __syncthreads();
        const int g = n - k;                            // rows evicted
        // rows behind the visual segment that have to close up; none when the tail keeps its place
        const int r = a.tail_start ? 0 : len - (a.sys_len + n);
        int m = 0;                                      // moves inside the visual segment
        if (a.mode == ST3_HOLE_FILL) {
            int base_h = 0, base_f = 0;
            for (int p0 = 0; p0 < n_pad; p0 += kSelThreads) {
                const int p = p0 + tid;
                const bool kept = p < n && flag_at(sm, p);
                const bool hole = p < k && !kept;
                const bool fill = p >= k && kept;
                int packed = (hole ? 1 : 0) | (fill ? (1 << 16) : 0);
                int incl = block_incl_scan(packed, sm);
                if (hole) mv[2 * (base_h + (incl & 0xffff) - 1)] = a.sys_len + p;
                if (fill) mv[2 * (base_f + (incl >> 16) - 1) + 1] = a.sys_len + p;
                __syncthreads();
                if (tid == kSelThreads - 1) sm.red = incl;
                __syncthreads();
                base_h += sm.red & 0xffff;
                base_f += sm.red >> 16;
            }
            m = min(base_h, base_f);                    // equal when the ids are distinct
            __syncthreads();                            // move list visible to the whole block
            for (int i = tid; i < m; i += kSelThreads) {    // sources >= k, destinations < k: disjoint
                int dst = mv[2 * i] - a.sys_len, src = mv[2 * i + 1] - a.sys_len;
                scores[dst] = scores[src];
                ids[dst] = ids[src];
            }
            // refill the vacated end of the segment [k, n): from the END of the cache when at least
            // g rows follow the segment, else all r following rows move down.  Either way sources
            // and destinations are disjoint: r >= g -> src >= len-g >= sys+n; r < g -> dst < sys+k+r < sys+n.
            const int cnt = min(g, r);
            const int src0 = (r >= g) ? len - g : a.sys_len + n;
            for (int j = tid; j < cnt; j += kSelThreads) {
                mv[2 * (m + j)] = a.sys_len + k + j;
                mv[2 * (m + j) + 1] = src0 + j;
            }
            moves_left = m + cnt;
            if (a.inline_apply) {
                __syncthreads();
                copy_rows_all_strips(a, b, mv, 0, m);       // holes <- surviving tail of the segment
                __syncthreads();                            // those reads are done before [k, n) is overwritten
                copy_rows_all_strips(a, b, mv, m, cnt);
                moves_left = 0;
            }
        } else {
            // first hole = number of leading kept positions
            int fh = n;
            for (int p = tid; p < n; p += kSelThreads)
                if (!flag_at(sm, p)) { fh = p; break; }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) fh = min(fh, __shfl_xor(fh, off));
            if (tid % kWave == 0) sm.wave_tot[tid / kWave] = fh;
            __syncthreads();
            fh = min(min(sm.wave_tot[0], sm.wave_tot[1]), min(sm.wave_tot[2], sm.wave_tot[3]));
            __syncthreads();
            int base = 0;
            for (int p0 = 0; p0 < n_pad; p0 += kSelThreads) {
                const int p = p0 + tid;
                const bool kept = p < n && flag_at(sm, p);
                float sv = 0.f; int32_t iv = 0;
                if (kept) { sv = scores[p]; iv = ids[p]; }
                int incl = block_incl_scan(kept ? 1 : 0, sm);       // contains barriers: loads precede stores
                const int rank = base + incl - 1;
                if (kept && p > fh) {
                    scores[rank] = sv; ids[rank] = iv;
                    mv[2 * (rank - fh)] = a.sys_len + rank;
                    mv[2 * (rank - fh) + 1] = a.sys_len + p;
                }
                __syncthreads();
                if (tid == kSelThreads - 1) sm.red = incl;
                __syncthreads();
                base += sm.red;
            }
            m = k - fh;
            for (int j = tid; j < r; j += kSelThreads) {
                mv[2 * (m + j)] = a.sys_len + k + j;
                mv[2 * (m + j) + 1] = a.sys_len + n + j;
            }
            moves_left = m + r;
        }
        new_len = a.tail_start ? len : len - g;
        if (tid == 0) a.vis_len[b] = k;
    }
    if (tid == 0) {
        a.move_cnt[b] = moves_left;
        a.kv_len[b] = new_len;
    }
}

// ---- host side (defined in st3_select.hip) --------------------------------------------------
// Fills the plan arguments for one layer; needs_apply tells whether evict_apply_kernel must run
// after the plan (evictions too large for the plan workgroup to move, or STABLE mode).
// kv->k may be null (a layer that caches V only).  mass_workspace (null: `workspace`) is the
// workspace whose attend launch left the logits the mass is finished from - a lazy layer's
// source - and mass_capacity that cache's capacity.  batched: the plan will share its launch with
// the plans of other layers (decides how many row moves the plan workgroup does itself).
st3_status build_evict_args(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                            float* score_col, int32_t* id_col, int64_t col_stride, int32_t keep_count, int32_t mode,
                            void* workspace, size_t workspace_bytes, int appended, float* mass_dst,
                            int64_t mass_stride, EvictArgs& ea, bool& needs_apply, bool batched,
                            const void* mass_workspace = nullptr, int32_t mass_capacity = 0);
void launch_evict_plan(const EvictArgs& ea, int B, hipStream_t st);
constexpr int kPlanBatch = 16;     // plans that fit the kernel-argument block by value
// Plans of n layers (device work of one decode step) with one launch per kPlanBatch layers.
void launch_evict_plan_batch(const EvictArgs* plans, int n, int B, hipStream_t st);
// The same for plans that the layers' attention launches have left in device memory (PlanStash):
// stashed[i] is where layer i's copy of plans[i] lies; one launch per kPlanTableMax layers.
constexpr int kPlanTableMax = 64;
static_assert(sizeof(EvictArgs) <= kPlanStashWords * sizeof(uint32_t), "a layer's plan must fit the stash");
void launch_evict_plan_table(const EvictArgs* const* stashed, const EvictArgs* plans, int n, int B, hipStream_t st);
void launch_evict_apply(const EvictArgs& ea, int B, hipStream_t st);

}  // namespace st3
