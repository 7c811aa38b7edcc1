// Decode attention over a ragged KV cache (Eq. 2 with a single query row that follows every
// cached key) with the visual mass of Sec. 3.2, plus KV append.
//
// decode_attend_kernel streams K and V exactly once.  Each (b,h) strip is cut into `nsplit`
// chunks (one workgroup each); nsplit is 1 as soon as B*H alone fills the chip and the strip is no
// longer than the logit staging area, and then the workgroup writes the finished output row itself.  With nsplit > 1 the workgroups leave
// un-normalised partials that decode_finish_kernel merges in chunk order.  For the visual mass the
// attend kernel saves the scaled logits of the visual keys (collected in LDS, written out as whole
// lines at the end of the workgroup) and every chunk's (max, sum); turning
// them into probabilities and adding them over heads - in head order, so the sum is the same on
// every run - is done by finish_mass(): in decode_finish_kernel for the stand-alone call, and by
// the layer's eviction-plan workgroup in the fused step (it needs the scores only then).
// The token being appended is read from k_new/v_new as cache row kv_len[b] by the workgroup that
// owns the end of the strip, which also stores it into the cache; kv_len itself is bumped by the
// eviction plan that follows the attention.
// (Letting that plan ride in spare workgroups of the next layer's attend launch was measured and
// dropped: a plan workgroup is a chain of dependent memory round trips that outlasts the attend
// launch and halves the streaming rate of the compute unit it sits on.)
//
// No kernel here communicates between workgroups of one launch: device-scope fences cost a
// write-back and invalidate of the XCD-private L2 on this part and were measured to be ruinous.
#include <hip/hip_ext.h>

#include <atomic>
#include <cmath>
#include <utility>

#include "st3_common.h"
#include "st3_attend.h"
#include "st3_decode.h"

#ifndef ST3_DECODE_THREADS
#define ST3_DECODE_THREADS 256      // threads per workgroup of the attend kernel
#endif
#ifndef ST3_DECODE_MIN_BLOCKS
#define ST3_DECODE_MIN_BLOCKS 2     // workgroups per CU the register budget must allow
#endif

namespace st3 {

bool profile_take(hipEvent_t* start, hipEvent_t* stop);     // st3_api.hip

namespace {

constexpr int kDecodeThreads = ST3_DECODE_THREADS;
constexpr int kDecodeWaves = kDecodeThreads / kWave;

struct DecodeArgs {
    const void* q;
    void* k;
    void* v;
    int64_t stride_b, stride_h, stride_t;
    const int32_t* kv_len;
    const int32_t* vis_len;
    const int32_t* tail_start;  // [B] or null (the tail follows the visual rows directly)
    int32_t B, sys_len, max_vis, max_kv, H, nsplit, nsplit_cap, chunk, capacity;
    int32_t hint_base, hint_gap;    // the host's guess at the layout of a fixed-tail cache (INT_MAX, 0: none)
    int32_t defer;          // 1: the mass of this call is finished by the eviction plan that follows; mark it pending
    int32_t keep_all_logits;  // 1: keep the logit of every key (a lazy layer will ask for them), else visual only
    float scale_l2;
    const float* k_scale;   // [B*H] value of one K code unit (E4M3 caches; null: 1)
    const float* v_scale;   // [B*H] likewise for V
    float* part_o;          // [B,H,nsplit_cap,D]   (nsplit > 1 only)
    float* part_ml;         // [B,H,nsplit_cap,2]
    float* logits;          // [B,H,capacity]; null when no mass is wanted
    int32_t stage_rows;     // floats of LDS in which a workgroup collects the logits it keeps (0 when it keeps none)
    int32_t* pending;       // [B][4]: {mass still to be finished | rows attended << 1, nsplit, chunk, logits of this call present}
    const void* k_new;      // [B,H,D] rows of the token being appended (null: none); the cache row
    const void* v_new;      //         kv_len[b] is then taken from here and written to the cache
    void* out;              // [B,H,D]
};

// Workgroup (0,0,0) of a launch leaves the stash words in the workspace (plain vector stores).  The stash is a kernel
// parameter of its own, behind the argument struct, so that the struct's fields keep their places in the argument block.
__device__ __forceinline__ void leave_stash(const PlanStash& st) {
    if (st.dst != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x < kPlanStashWords)
        st.dst[threadIdx.x] = st.w[threadIdx.x];
}

template <typename T>
__device__ __forceinline__ void store_out(void* out, int64_t idx, float o) {
    if (sizeof(T) == 4) reinterpret_cast<float*>(out)[idx] = o;
    else reinterpret_cast<uint16_t*>(out)[idx] = (uint16_t)f32_to_bf16_bits(o);
}

// This lane's 16-byte slice of a new token's row, in the format of the cache it is going into
// (lane map of RowMap<KT, D>): a plain copy when the cache holds elements of T, the E4M3 quantiser
// otherwise.  What the attention then reads is exactly what later steps will find in the cache.
template <typename T, typename KT, int D>
struct NewRow {
    static __device__ __forceinline__ u32x4_t load(const T* row, int lane, float) {
        using M = RowMap<KT, D>;
        return *reinterpret_cast<const u32x4_t*>(row + (lane % M::LPR) * M::EPL);
    }
};
template <typename T, int D>
struct NewRow<T, e4m3_t, D> {
    static __device__ __forceinline__ u32x4_t load(const T* row, int lane, float scale) {
        float f[16];
        load_row_slice<T, e4m3_t, D>(row, lane, f);
        u32x4_t r;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            r[i] = quantize_e4m3(f[4 * i], scale) | (quantize_e4m3(f[4 * i + 1], scale) << 8) |
                   (quantize_e4m3(f[4 * i + 2], scale) << 16) | (quantize_e4m3(f[4 * i + 3], scale) << 24);
        return r;
    }
};

// grid (nsplit, H, B).  T: element type of q, k_new, v_new and out; KT: element type of the cache.
template <typename T, typename KT, int D, int U>
__global__ __launch_bounds__(kDecodeThreads, ST3_DECODE_MIN_BLOCKS)
__attribute__((amdgpu_waves_per_eu(ST3_DECODE_MIN_BLOCKS, ST3_DECODE_MIN_BLOCKS)))    // do not spill to reach a third wave
void decode_attend_kernel(DecodeArgs a, PlanStash stash) {
    using M = RowMap<KT, D>;
    constexpr int EPL = M::EPL, LPR = M::LPR, TILE = U * M::RPL;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int c0 = split * a.chunk;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int64_t bh = (int64_t)b * a.H + h;
    const T* qrow = reinterpret_cast<const T*>(a.q) + bh * D;
    KT* kbase = reinterpret_cast<KT*>(a.k) + b * a.stride_b + h * a.stride_h;
    KT* vbase = reinterpret_cast<KT*>(a.v) + b * a.stride_b + h * a.stride_h;
    if (a.max_kv > 0 && c0 >= a.max_kv) return;     // (the host launches no such chunk; the early loads below rely on it)
    // The first tile's loads go out before the sequence length has arrived: the host bound keeps
    // them inside the strip (rows the length later rules out are masked when the tile is consumed).
    // Takes one dependent memory round trip off the front of every workgroup.  Where the cache keeps
    // a gap behind its visual segment the rows are placed by the host's guess at it.
    uint4 kr[U], vr[U];
    const RowShift guess{a.hint_base, a.hint_gap};
    issue_tile_within<KT, D, U, true>(kbase, vbase, a.stride_t, c0 + wave * TILE, c0 + a.chunk,
                                     a.max_kv - (a.k_new != nullptr ? 1 : 0), c0, lane, kr, vr, guess);
    float qf[EPL];
    load_row_slice<T, KT, D>(qrow, lane, qf);
    // a code unit of K is worth k_scale: folded into the logit scale; V's goes onto the output
    const float k_unit = a.k_scale ? a.k_scale[bh] : 1.0f, v_unit = a.v_scale ? a.v_scale[bh] : 1.0f;
    const float scale_l2 = a.scale_l2 * k_unit;
    // the row being appended sits at index kv_len[b]; never trust a device length past the host bound
    const int len_phys = min(a.kv_len[b] + (a.k_new != nullptr ? 1 : 0), a.max_kv);
    // `len` and every row index below are in the gap-free numbering (a cache with a fixed tail keeps
    // dead rows between the visual segment and the tail); `sh` maps a row to where it is stored
    const SeqLayout lay = seq_layout(a.sys_len, a.vis_len[b], a.max_vis, len_phys, a.tail_start, b);
    const int len = lay.vlen;
    const RowShift sh = lay.shift();
    leave_stash(stash);
    if (split == 0 && h == 0 && tid == 0 && a.pending != nullptr) {
        // bit 0: the mass of this launch is still to be finished; above it: the rows this launch attends over
        a.pending[b * 4 + 0] = ((a.logits != nullptr && len > 0 && a.defer) ? 1 : 0) | (max(len, 0) << 1);
        a.pending[b * 4 + 1] = a.nsplit;
        a.pending[b * 4 + 2] = a.chunk;
        a.pending[b * 4 + 3] = (a.logits != nullptr && len > 0 && a.keep_all_logits) ? 1 : 0;
    }
    if (len <= 0) {                                  // empty sequence: out = 0, no mass
        if (split == 0 && tid < D) store_out<T>(a.out, bh * D + tid, 0.f);
        return;
    }
    if (c0 >= len) return;
    const int c1 = min(c0 + a.chunk, len);

    WaveState<EPL> st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) st.acc[e] = 0.f;

    // Scaled logits kept for later: those of the visual keys become the mass; a layer with lazy
    // followers (QK heredity, Eq. 6) keeps the logit of EVERY key for them.  Keeping all of them
    // always was measured at +5 % on this kernel (4 bytes stored against 512 read per key, but as
    // partial-line writes), so it is done only where it is needed.  Index = cache row either way.
    float* lg = a.logits ? a.logits + bh * a.capacity : nullptr;
    const int vis_lo = a.keep_all_logits ? 0 : a.sys_len;
    const int vis_hi = a.keep_all_logits ? len : a.sys_len + lay.nv;
    if (lg) lg += vis_lo;           // the wave loop indexes by (row - vis_lo)
    // this workgroup owns the appended row (stored at the physical end, which a fixed tail must have reached)
    const bool has_new = a.k_new != nullptr && c1 == len && len_phys - 1 >= lay.base + lay.gap;
    const int c1_cached = has_new ? c1 - 1 : c1;
    // the appended token's row is fetched now and used after the cached rows: off the critical path
    u32x4_t kn_raw = {0, 0, 0, 0}, vn_raw = {0, 0, 0, 0};       // native vectors: the uint4 class would live in scratch
    if (has_new && wave == 0) {
        kn_raw = NewRow<T, KT, D>::load(reinterpret_cast<const T*>(a.k_new) + bh * D, lane, k_unit);
        vn_raw = NewRow<T, KT, D>::load(reinterpret_cast<const T*>(a.v_new) + bh * D, lane, v_unit);
    }
    // waves take the tiles of the chunk round-robin, so all four stay busy to the end
    // the early tile placed its rows by the host's guess: fetch it again if that put a row this
    // sequence attends to in the wrong place (a sequence that differs from the guess, in a tile that
    // reaches behind its visual segment or the guessed one)
    {
        const int tile_end = min(c0 + wave * TILE + TILE, c1_cached);
        const bool same = lay.gap == guess.gap && (lay.gap == 0 || lay.base == guess.split_row);
        const bool in_front = tile_end <= lay.base && (guess.gap == 0 || tile_end <= guess.split_row);
        if (!same && !in_front)
            issue_tile<KT, D, U, true>(kbase, vbase, a.stride_t, c0 + wave * TILE, c1_cached, c0, lane, kr, vr, sh);
    }
    // rows of the early tile that the length rules out came from beyond the sequence: their V may
    // hold anything (NaN included), and 0 * NaN would poison the accumulator
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (c0 + wave * TILE + u * M::RPL + lane / LPR >= c1_cached) vr[u] = make_uint4(0, 0, 0, 0);
    // The logits this workgroup keeps (rows [lg_lo, lg_hi) of its chunk) are collected in LDS and leave
    // as whole lines after the waves have merged: stored one by one from the loop (16 bytes per wave
    // and tile) they cost 2 us of a 66 us launch at the 13B shape.  The launcher cuts strips so that a
    // chunk's rows fit the staging area (kLogitStageMaxRows) whenever logits are kept.
    extern __shared__ float sm_lg[];
    const int lg_lo = max(c0, vis_lo), lg_hi = min(c1, vis_hi);
    float* lg_stage = lg != nullptr ? sm_lg : nullptr;
    wave_attend_primed<KT, D, U, true>(qf, kbase, vbase, a.stride_t, c0 + wave * TILE, c1_cached, kDecodeWaves * TILE,
                                       c0, scale_l2, lane, st, lg_stage, lg_lo, vis_hi, kr, vr, sh);
    if (has_new && wave == 0) {
        wave_attend_row<KT, D>(qf, make_uint4(kn_raw.x, kn_raw.y, kn_raw.z, kn_raw.w),
                               make_uint4(vn_raw.x, vn_raw.y, vn_raw.z, vn_raw.w), len - 1, scale_l2, lane, st, lg_stage, lg_lo,
                               vis_hi);
        if (lane < 2 * LPR) {                       // store the row into the cache: lanes [0,LPR) K, [LPR,2*LPR) V
            KT* dst = (lane < LPR ? kbase : vbase) + (int64_t)(len_phys - 1) * a.stride_t + (lane % LPR) * EPL;
            *reinterpret_cast<u32x4_t*>(dst) = lane < LPR ? kn_raw : vn_raw;
        }
    }
    finish_wave<KT, D>(st);

    __shared__ float sm_acc[kDecodeWaves][D];
    __shared__ float sm_m[kDecodeWaves], sm_l[kDecodeWaves];
    if (lane < LPR) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sm_acc[wave][lane * EPL + e] = st.acc[e];
    }
    if (lane == 0) { sm_m[wave] = st.m; sm_l[wave] = st.l; }
    __syncthreads();
    if (lg != nullptr) {
        for (int i = tid; i < lg_hi - lg_lo; i += kDecodeThreads) lg[lg_lo - vis_lo + i] = sm_lg[i];
    }
    if (tid < D) {
        float m = sm_m[0];
#pragma unroll
        for (int w = 1; w < kDecodeWaves; ++w) m = fmaxf(m, sm_m[w]);   // finite: the chunk is not empty
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            float f = exp2_fast(sm_m[w] - m);           // wave without rows: exp2(-inf) = 0
            o = fmaf(sm_acc[w][tid], f, o);
            l = fmaf(sm_l[w], f, l);
        }
        const int64_t slot = bh * a.nsplit_cap + split;
        if (a.nsplit == 1) store_out<T>(a.out, bh * D + tid, o / l * v_unit);
        else a.part_o[slot * D + tid] = o * v_unit;
        if (tid == 0) { a.part_ml[slot * 2] = m; a.part_ml[slot * 2 + 1] = l; }
    }
}

// ---------------------------------------------------------------------------------------------
// Lazy layer (QK heredity, Eq. 6 / Alg. 2): o = sum_j p_j V[j] with the probabilities p of the
// SOURCE layer's attention of the same step, rebuilt from the logits and chunk (max, sum) pairs
// that the source's attend launch left in its workspace.  Streams V once: half the bytes.
// ---------------------------------------------------------------------------------------------
struct InheritArgs {
    void* v;
    int64_t stride_b, stride_h, stride_t;
    const int32_t* kv_len;
    const int32_t* vis_len;
    const int32_t* tail_start;  // [B] or null
    int32_t B, max_kv, H, nsplit, nsplit_cap, chunk, sys_len, max_vis;
    const float* src_logits;    // [B,H,src_capacity]
    const float* src_part_ml;   // [B,H,src_nsplit_cap,2]
    const int32_t* src_pending; // [B][4]
    int32_t src_capacity, src_nsplit_cap;
    float* part_o;              // [B,H,nsplit_cap,D]   (nsplit > 1 only)
    const void* v_new;          // [B,H,D] value row of the token being appended (null: none)
    const float* v_scale;       // [B*H] value of one V code unit (E4M3 caches; null: 1)
    void* out;
};

// One wave over the tiles of U*RPL value rows starting at r0, r0+step, ... below r1; next tile's
// loads are issued before the current tile is consumed.
template <typename T, int D, int U>
__device__ __forceinline__ void wave_inherit(const T* vbase, int64_t stride_t, int r0, int r1, int step, int safe_row,
                                             const float* lg, float m, float rl, int lane, float* acc,
                                             const RowShift sh) {
    using M = RowMap<T, D>;
    constexpr int EPL = M::EPL, LPR = M::LPR, RPL = M::RPL;
    const int grp = lane / LPR;
    const int64_t col = (int64_t)(lane % LPR) * EPL;
    if (r0 >= r1) return;
    u32x4_t vr[U], vn[U];
    float sr[U], sn[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int row = r0 + u * RPL + grp;
        const int rr = row < r1 ? row : safe_row;
        vr[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(vbase + (int64_t)sh.physical(rr) * stride_t + col));
        sr[u] = lg[rr];
    }
    for (int t0 = r0; t0 < r1; t0 += step) {
        const int tn = t0 + step;
        if (tn < r1) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = tn + u * RPL + grp;
                const int rr = row < r1 ? row : safe_row;
                vn[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(vbase + (int64_t)sh.physical(rr) * stride_t + col));
                sn[u] = lg[rr];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = t0 + u * RPL + grp;
            const float p = row < r1 ? exp2_fast(sr[u] - m) * rl : 0.f;
            float vf[EPL];
            ElemTraits<T>::unpack(make_uint4(vr[u].x, vr[u].y, vr[u].z, vr[u].w), vf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
        }
        if (tn < r1) {
#pragma unroll
            for (int u = 0; u < U; ++u) { vr[u] = vn[u]; sr[u] = sn[u]; }
        }
    }
}

// grid (nsplit, H, B)
template <typename T, typename KT, int D, int U>
__global__ __launch_bounds__(kDecodeThreads, ST3_DECODE_MIN_BLOCKS) void decode_inherit_kernel(InheritArgs a, PlanStash stash) {
    using M = RowMap<KT, D>;
    constexpr int EPL = M::EPL, LPR = M::LPR, TILE = U * M::RPL;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    leave_stash(stash);
    const int len_phys = min(a.kv_len[b] + (a.v_new != nullptr ? 1 : 0), a.max_kv);
    // rows are numbered without the gap a fixed-tail cache keeps behind its visual segment, as in the
    // source layer's attend launch (same lengths, same layout): its logits are indexed the same way
    const SeqLayout lay = seq_layout(a.sys_len, a.vis_len[b], a.max_vis, len_phys, a.tail_start, b);
    const int len = lay.vlen;
    const int c0 = split * a.chunk;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int64_t bh = (int64_t)b * a.H + h;
    const bool have = a.src_pending[b * 4 + 3] != 0;        // the source attended a non-empty sequence
    if (len <= 0 || !have) {                                // nothing to inherit: out = 0
        if (split == 0 && tid < D) store_out<T>(a.out, bh * D + tid, 0.f);
        if (len > 0 && a.nsplit > 1 && c0 < len && tid < D) a.part_o[(bh * a.nsplit_cap + split) * D + tid] = 0.f;
        return;
    }
    if (c0 >= len) return;
    const int c1 = min(c0 + a.chunk, len);
    // the source row's maximum and sum from its chunk pairs, in chunk order (every thread alike)
    const int s_nsplit = min(a.src_pending[b * 4 + 1], a.src_nsplit_cap);
    const int s_chunk = max(a.src_pending[b * 4 + 2], 32);
    const int s_ns = min((len + s_chunk - 1) / s_chunk, s_nsplit);
    const float* ml = a.src_part_ml + bh * a.src_nsplit_cap * 2;
    float m = ml[0];
    for (int s = 1; s < s_ns; ++s) m = fmaxf(m, ml[2 * s]);
    float l = 0.f;
    for (int s = 0; s < s_ns; ++s) l = fmaf(ml[2 * s + 1], exp2_fast(ml[2 * s] - m), l);
    const float rl = 1.0f / l;

    KT* vbase = reinterpret_cast<KT*>(a.v) + b * a.stride_b + h * a.stride_h;
    const float* lg = a.src_logits + bh * a.src_capacity;
    const float v_unit = a.v_scale ? a.v_scale[bh] : 1.0f;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    const bool has_new = a.v_new != nullptr && c1 == len && len_phys - 1 >= lay.base + lay.gap;
    const int c1_cached = has_new ? c1 - 1 : c1;
    wave_inherit<KT, D, U>(vbase, a.stride_t, c0 + wave * TILE, c1_cached, kDecodeWaves * TILE, c0, lg, m, rl, lane, acc,
                           lay.shift());
    if (has_new && wave == 0 && lane < LPR) {
        const u32x4_t raw = NewRow<T, KT, D>::load(reinterpret_cast<const T*>(a.v_new) + bh * D, lane, v_unit);
        const float p = exp2_fast(lg[len - 1] - m) * rl;
        float vf[EPL];
        ElemTraits<KT>::unpack(make_uint4(raw.x, raw.y, raw.z, raw.w), vf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
        *reinterpret_cast<u32x4_t*>(vbase + (int64_t)(len_phys - 1) * a.stride_t + lane * EPL) = raw;
    }
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], off);
    }
    __shared__ float sm_acc[kDecodeWaves][D];
    if (lane < LPR) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sm_acc[wave][lane * EPL + e] = acc[e];
    }
    __syncthreads();
    if (tid < D) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) o += sm_acc[w][tid];
        if (a.nsplit == 1) store_out<T>(a.out, bh * D + tid, o * v_unit);
        else a.part_o[(bh * a.nsplit_cap + split) * D + tid] = o * v_unit;
    }
}

struct FinishArgs {
    const float* part_o;
    const float* part_ml;
    const float* logits;
    const int32_t* kv_len;
    const int32_t* vis_len;
    const int32_t* tail_start;  // [B] or null
    int32_t H, nsplit, nsplit_cap, chunk, capacity, max_vis, max_kv, sys_len;
    int32_t plain_sum;      // 1: the partial outputs are already normalised, just add them (lazy layers)
    int32_t appended;       // 1: the attend kernel took one more row than kv_len[b] says (the token being appended)
    void* out;              // null: outputs already written (nsplit == 1)
    float* mass;            // null: no mass
    int64_t mass_stride;
};

// grid (out_blocks + mass_blocks, B), 256 threads.  Blocks x < H (when out != null) merge the
// chunk partials of head x; the rest produce 256 mass entries each.
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_finish_kernel(FinishArgs a) {
    const int b = blockIdx.y, tid = threadIdx.x;
    const SeqLayout lay = seq_layout(a.sys_len, a.vis_len[b], a.max_vis, min(a.kv_len[b] + a.appended, a.max_kv),
                                     a.tail_start, b);
    const int len = lay.vlen;                           // rows the attend launch saw
    const int ns = len > 0 ? min((len + a.chunk - 1) / a.chunk, a.nsplit) : 0;
    const int out_blocks = a.out ? a.H : 0;
    if ((int)blockIdx.x < out_blocks) {
        const int h = blockIdx.x;
        const int64_t bh = (int64_t)b * a.H + h;
        if (tid >= D || ns == 0) return;                // empty sequence: the attend kernel wrote zeros
        if (a.plain_sum) {
            float o = 0.f;
            for (int s = 0; s < ns; ++s) o += a.part_o[(bh * a.nsplit_cap + s) * D + tid];   // chunk order
            store_out<T>(a.out, bh * D + tid, o);
            return;
        }
        const float* ml = a.part_ml + bh * a.nsplit_cap * 2;
        float m = ml[0];
        for (int s = 1; s < ns; ++s) m = fmaxf(m, ml[2 * s]);
        float l = 0.f, o = 0.f;
        for (int s = 0; s < ns; ++s) {                  // fixed order: chunk 0, 1, ...
            float f = exp2_fast(ml[2 * s] - m);
            l = fmaf(ml[2 * s + 1], f, l);
            o = fmaf(a.part_o[(bh * a.nsplit_cap + s) * D + tid], f, o);
        }
        store_out<T>(a.out, bh * D + tid, o / l);
        return;
    }
    if (a.mass == nullptr) return;
    __shared__ float sm_m[1024], sm_rl[1024];
    const int nv = lay.nv;
    head_norms(a.part_ml, b, a.H, ns, a.nsplit_cap, sm_m, sm_rl);
    const int j0 = ((int)blockIdx.x - out_blocks) * 256;
    finish_mass(a.logits + a.sys_len, b, a.H, a.capacity, sm_m, sm_rl, j0, min(j0 + 256, nv),
                a.mass + (int64_t)b * a.mass_stride);
}

struct AppendArgs {
    void* k;
    void* v;
    int64_t stride_b, stride_h, stride_t;
    const void* k_new;
    const void* v_new;
    const int32_t* kv_len;
    const float* k_scale;
    const float* v_scale;
    int32_t H, capacity;
};

// grid (H, B), 64 threads: lanes [0, LPR) write the K row, lanes [LPR, 2*LPR) the V row.
template <typename T, typename KT, int D>
__global__ __launch_bounds__(64) void append_kernel(AppendArgs a) {
    using M = RowMap<KT, D>;
    const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const int row = a.kv_len[b];
    if (row < 0 || row >= a.capacity || lane >= 2 * M::LPR) return;
    const bool is_v = lane >= M::LPR;
    if (!is_v && a.k == nullptr) return;                // a layer that caches V only
    const int64_t bh = (int64_t)b * a.H + h;
    const float* sc = is_v ? a.v_scale : a.k_scale;
    const T* src = reinterpret_cast<const T*>(is_v ? a.v_new : a.k_new) + bh * D;
    const u32x4_t raw = NewRow<T, KT, D>::load(src, lane % M::LPR, sc ? sc[bh] : 1.0f);
    KT* dst = reinterpret_cast<KT*>(is_v ? a.v : a.k) + b * a.stride_b + h * a.stride_h + row * a.stride_t +
              (lane % M::LPR) * M::EPL;
    *reinterpret_cast<u32x4_t*>(dst) = raw;
}

// Rows [0, n) of a [B,H,n,D] tensor of T into rows [0, n) of one half of a cache, in its format.
struct QuantArgs {
    const void* src;
    int64_t s_sb, s_sh, s_st;       // elements of T
    void* dst;
    int64_t d_sb, d_sh, d_st;       // cache elements
    const float* scale;             // [B*H] or null
    int32_t H, n;
};

// grid (ceil(n / rows per block), H, B), 256 threads: LPR lanes per row.
template <typename T, typename KT, int D>
__global__ __launch_bounds__(256) void quantize_rows_kernel(QuantArgs a) {
    using M = RowMap<KT, D>;
    const int h = blockIdx.y, b = blockIdx.z;
    const int row = blockIdx.x * (256 / M::LPR) + threadIdx.x / M::LPR;
    if (row >= a.n) return;
    const int64_t bh = (int64_t)b * a.H + h;
    const T* src = reinterpret_cast<const T*>(a.src) + b * a.s_sb + h * a.s_sh + row * a.s_st;
    const u32x4_t raw = NewRow<T, KT, D>::load(src, threadIdx.x % M::LPR, a.scale ? a.scale[bh] : 1.0f);
    KT* dst = reinterpret_cast<KT*>(a.dst) + b * a.d_sb + h * a.d_sh + row * a.d_st + (threadIdx.x % M::LPR) * M::EPL;
    *reinterpret_cast<u32x4_t*>(dst) = raw;
}

__global__ void bump_len_kernel(int32_t* kv_len, int32_t B, int32_t capacity) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B && kv_len[b] >= 0 && kv_len[b] < capacity) kv_len[b] += 1;
}

// ---------------------------------------------------------------------------------------------
// Tile size (U = 16-byte loads of K, and of V, in flight per lane and tile; a wave-wide load is 1 KB).
// While every workgroup of a launch is resident at once, a tile of 8 KB per wave is the fastest for
// two- and four-byte caches (U = 4: 16 bf16 rows; room for four workgroups per compute unit, short
// strips pipelined in finer steps: 5-9 % faster than U = 8 at B*H = 40 ... 640 strips), 6 KB for E4M3
// (U = 3: 24 rows).  With more workgroups than the device holds, what counts is how full the last
// round of workgroups is: B*H = 1280 bf16 strips are 1.25 rounds at U = 4 (slowest), 1.67 at U = 6,
// 2.5 at U = 8, and fit at once at U = 1 (66 registers, seven workgroups per unit: fastest, though
// much the slowest build for small launches).  So the launcher asks the runtime how many workgroups
// of each build the device holds and takes the build that wastes least of its last round; the
// candidate lists below are in order of preference for ties.
// ---------------------------------------------------------------------------------------------
// The current device's id when it indexes the per-device caches below, else -1 (then nothing is cached).
int current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

int compute_units(int dev) {
    static std::atomic<int> cached[kMaxDevices];    // 0 = not asked yet; a race only repeats the query
    if (dev >= 0 && cached[dev].load(std::memory_order_relaxed) != 0) return cached[dev].load(std::memory_order_relaxed);
    int n = 0;
    if (dev < 0 || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    if (dev >= 0) cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

// Workgroups of `kernel` (256 threads, no dynamic LDS) the current device holds at once; `cache` is
// the kernel's own array of one entry per device.
template <typename K>
int resident_workgroups(K kernel, std::atomic<int>* cache) {
    const int dev = current_device();
    if (dev >= 0 && cache[dev].load(std::memory_order_relaxed) != 0) return cache[dev].load(std::memory_order_relaxed);
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kDecodeThreads, 0) != hipSuccess || per_cu < 1)
        per_cu = 1;
    const int n = per_cu * compute_units(dev);
    if (dev >= 0) cache[dev].store(n, std::memory_order_relaxed);
    return n;
}

// Time of a launch of `items` equal workgroups on `slots` concurrent ones, relative to a launch whose
// last round is full.
inline double last_round_cost(int64_t items, int slots) {
    const double rounds = (double)items / (double)slots;
    return rounds <= 1.0 ? 1.0 : std::ceil(rounds) / rounds;
}

// Index of the cheapest of n candidates (ordered by preference: the first wins ties).
inline int cheapest(const double* cost, int n) {
    int best = 0;
    for (int i = 1; i < n; ++i)
        if (cost[i] < cost[best] - 1e-9) best = i;
    return best;
}

template <typename T, typename KT, int D, int U>
void launch_attend_u(const DecodeArgs& da, const PlanStash& ps, int B, hipStream_t st) {
    const dim3 grid(da.nsplit, da.H, B);
    const size_t lds = (size_t)da.stage_rows * sizeof(float);       // dynamic LDS: the logit staging area
    hipEvent_t e0, e1;
    if (profile_take(&e0, &e1))     // timed launch: the events receive the kernel's own start and end
        hipExtLaunchKernelGGL((decode_attend_kernel<T, KT, D, U>), grid, dim3(kDecodeThreads), lds, st, e0, e1, 0, da, ps);
    else
        decode_attend_kernel<T, KT, D, U><<<grid, kDecodeThreads, lds, st>>>(da, ps);
}

// Takes the cheapest of the builds Us... (in order of preference) for this launch.
template <typename T, typename KT, int D, int... Us>
void launch_attend_best(const DecodeArgs& da, const PlanStash& ps, int B, hipStream_t st, std::integer_sequence<int, Us...>) {
    constexpr int N = sizeof...(Us);
    static std::atomic<int> slots[N][kMaxDevices];  // resident workgroups of each build, per device
    const int us[N] = {Us...};
    const int g_forced_tile = debug_state().attend_tile;    // 0 unless the debug block is enabled
    if (g_forced_tile != 0 && ((g_forced_tile == Us) || ...)) {
        ((g_forced_tile == Us ? (launch_attend_u<T, KT, D, Us>(da, ps, B, st), 0) : 0), ...);
        return;
    }
    const int64_t items = (int64_t)da.nsplit * da.H * B;
    double cost[N];
    int i = 0;
    ((cost[i] = last_round_cost(items, resident_workgroups(decode_attend_kernel<T, KT, D, Us>, slots[i])), ++i), ...);
    const int pick = us[cheapest(cost, N)];
    ((pick == Us ? (launch_attend_u<T, KT, D, Us>(da, ps, B, st), 0) : 0), ...);
}

template <typename T, typename KT, int D>
void launch_attend(const DecodeArgs& da, const PlanStash& ps, int B, hipStream_t st) {
    if constexpr (sizeof(KT) == 1) launch_attend_best<T, KT, D>(da, ps, B, st, std::integer_sequence<int, 3, 4, 1>{});
    else launch_attend_best<T, KT, D>(da, ps, B, st, std::integer_sequence<int, 4, 6, 8, 1>{});
}

// The V-only kernel of lazy layers: 4 loads per lane and tile (4 KB per wave) were the fastest or
// within 2 % of it at every batch size and for both cache formats (8, 12 and 16 loads lose up to
// 17 % where the launch has more workgroups than fit at once; 2 loads lose at small batches).
template <typename T, typename KT, int D>
void launch_inherit(const InheritArgs& ia, const PlanStash& ps, int B, hipStream_t st) {
    decode_inherit_kernel<T, KT, D, 4><<<dim3(ia.nsplit, ia.H, B), kDecodeThreads, 0, st>>>(ia, ps);
}

template <typename T, int D>
void launch_finish(const FinishArgs& fa, int B, hipStream_t st) {
    const int blocks = (fa.out ? fa.H : 0) + (fa.mass ? (fa.max_vis + 255) / 256 : 0);
    if (blocks > 0) decode_finish_kernel<T, D><<<dim3(blocks, B), 256, 0, st>>>(fa);
}

template <typename T, typename KT, int D>
void launch_append(const AppendArgs& aa, int B, int32_t* kv_len, hipStream_t st) {
    append_kernel<T, KT, D><<<dim3(aa.H, B), 64, 0, st>>>(aa);
    bump_len_kernel<<<(B + 255) / 256, 256, 0, st>>>(kv_len, B, aa.capacity);
}

template <typename T, typename KT, int D>
void launch_quantize(const QuantArgs& qa, int B, hipStream_t st) {
    using M = RowMap<KT, D>;
    const int rpb = 256 / M::LPR;
    quantize_rows_kernel<T, KT, D><<<dim3((qa.n + rpb - 1) / rpb, qa.H, B), 256, 0, st>>>(qa);
}

// Launchers that depend on the cache element type: KT = T for plain caches, e4m3_t (bf16 I/O only,
// checked on the host) for E4M3 caches.
#define ST3_DISPATCH_KV(fn, shape, kv, ...)                                                                    \
    do {                                                                                                       \
        if ((kv)->format == ST3_KV_E4M3) {                                                                     \
            if ((shape)->head_dim == 128) fn<bf16_t, e4m3_t, 128>(__VA_ARGS__);                                \
            else fn<bf16_t, e4m3_t, 64>(__VA_ARGS__);                                                          \
        } else if ((shape)->dtype == ST3_BF16) {                                                               \
            if ((shape)->head_dim == 128) fn<bf16_t, bf16_t, 128>(__VA_ARGS__);                                \
            else fn<bf16_t, bf16_t, 64>(__VA_ARGS__);                                                          \
        } else {                                                                                               \
            if ((shape)->head_dim == 128) fn<float, float, 128>(__VA_ARGS__);                                  \
            else fn<float, float, 64>(__VA_ARGS__);                                                            \
        }                                                                                                      \
    } while (0)

#define ST3_DISPATCH(fn, shape, ...)                                                                   \
    do {                                                                                               \
        if ((shape)->dtype == ST3_BF16) {                                                              \
            if ((shape)->head_dim == 128) fn<bf16_t, 128>(__VA_ARGS__); else fn<bf16_t, 64>(__VA_ARGS__); \
        } else {                                                                                       \
            if ((shape)->head_dim == 128) fn<float, 128>(__VA_ARGS__); else fn<float, 64>(__VA_ARGS__);   \
        }                                                                                              \
    } while (0)

st3_status check_kv(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg, bool value_only = false) {
    if (!kv || !seg || (!kv->k && !value_only) || !kv->v || !seg->kv_len || !seg->vis_len) return ST3_ERR_INVALID_ARG;
    if (kv->capacity <= 0 || seg->sys_len < 0 || seg->max_vis_len < 0 || seg->max_kv_len < 0)
        return ST3_ERR_INVALID_ARG;
    if (seg->max_kv_len > kv->capacity) return ST3_ERR_INVALID_ARG;
    if (seg->sys_len + seg->max_vis_len > kv->capacity) return ST3_ERR_INVALID_ARG;
    if (kv->stride_t < s->head_dim || kv->stride_h < 0 || kv->stride_b < 0) return ST3_ERR_INVALID_ARG;
    if (kv->format != ST3_KV_PLAIN && kv->format != ST3_KV_E4M3) return ST3_ERR_INVALID_ARG;
    if (kv->format == ST3_KV_E4M3) {
        if (s->dtype != ST3_BF16) return ST3_ERR_UNSUPPORTED;
        if ((kv->k && !kv->k_scale) || !kv->v_scale) return ST3_ERR_INVALID_ARG;
    }
    const int eb = kv_elem_bytes(s, kv);
    if ((kv->k && !aligned16(kv->k)) || !aligned16(kv->v)) return ST3_ERR_INVALID_ARG;
    if ((kv->stride_t * eb) % 16 || (kv->stride_h * eb) % 16 || (kv->stride_b * eb) % 16)
        return ST3_ERR_INVALID_ARG;
    return ST3_OK;
}

}  // namespace

// Whether a launch over kv_len <= max_kv_len rows cuts its strips into chunks (partials to merge).
bool decode_is_split(const st3_attn_shape* shape, const st3_kv_layer* kv, int32_t max_kv_len) {
    const DecodeWs wl = decode_ws(shape->batch, shape->heads, shape->head_dim, kv->capacity);
    int nsplit = decode_nsplit(shape->batch, shape->heads, max_kv_len, kDecodeTargetWgsMerged);
    if (nsplit > wl.nsplit_cap) nsplit = wl.nsplit_cap;
    const int chunk = decode_chunk(max_kv_len, nsplit);
    return (max_kv_len + chunk - 1) / chunk > 1;
}

// Enqueues attention (+ the finish kernel when it is needed).  max_kv_len bounds the length the
// kernels will see (kv_len[b], plus one when a token is appended: k_new/v_new non-null).
// defer_mass: leave the head reduction of the mass to the eviction plan that follows.
st3_status enqueue_decode(const st3_attn_shape* shape, const void* q, const st3_kv_layer* kv,
                          const st3_segments* seg, int32_t max_kv_len, const void* k_new, const void* v_new,
                          void* out, float* vis_mass, int64_t mass_stride, bool want_mass, bool defer_mass,
                          bool keep_all_logits, void* workspace, size_t workspace_bytes, hipStream_t st,
                          bool defer_merge, const PlanStash* stash) {
    const int B = shape->batch, H = shape->heads, D = shape->head_dim;
    const DecodeWs wl = decode_ws(B, H, D, kv->capacity);
    if (workspace_bytes < wl.total) return ST3_ERR_WORKSPACE_TOO_SMALL;
    char* ws = reinterpret_cast<char*>(workspace);
    want_mass = want_mass && seg->max_vis_len > 0;
    DecodeArgs da{};
    da.q = q; da.k = kv->k; da.v = kv->v;
    da.stride_b = kv->stride_b; da.stride_h = kv->stride_h; da.stride_t = kv->stride_t;
    da.kv_len = seg->kv_len; da.vis_len = seg->vis_len; da.tail_start = seg->tail_start;
    da.B = B; da.sys_len = seg->sys_len; da.max_vis = seg->max_vis_len; da.max_kv = max_kv_len; da.H = H;
    da.hint_base = 0x7fffffff; da.hint_gap = 0;
    if (seg->tail_start != nullptr && seg->tail_start_hint > 0) {
        const int nv = std::max(0, std::min(seg->vis_len_hint, seg->max_vis_len));
        const int base = seg->sys_len + nv;
        const int ts = std::min(seg->tail_start_hint, kv->capacity);    // (keeps row + gap far from overflow)
        if (ts > base) { da.hint_base = base; da.hint_gap = ts - base; }
    }
    da.nsplit = decode_nsplit(B, H, max_kv_len, defer_merge ? kDecodeTargetWgsMerged : kDecodeTargetWgs);
    if (da.nsplit > wl.nsplit_cap) da.nsplit = wl.nsplit_cap;
    da.nsplit_cap = wl.nsplit_cap;
    da.chunk = decode_chunk(max_kv_len, da.nsplit);
    da.nsplit = (max_kv_len + da.chunk - 1) / da.chunk;         // rounding the chunk up to 32 rows can leave chunks empty
    if (da.nsplit < 1) da.nsplit = 1;
    da.capacity = kv->capacity;
    da.scale_l2 = scale_log2(shape);
    if (kv->format == ST3_KV_E4M3) { da.k_scale = kv->k_scale; da.v_scale = kv->v_scale; }
    da.part_o = reinterpret_cast<float*>(ws + wl.part_o);
    da.part_ml = reinterpret_cast<float*>(ws + wl.part_ml);
    da.logits = (want_mass || keep_all_logits) ? reinterpret_cast<float*>(ws + wl.logits) : nullptr;
    da.keep_all_logits = keep_all_logits ? 1 : 0;
    // a workgroup keeps at most this many logits: all rows of its chunk, or the visual ones (chunk <= kLogitStageMaxRows)
    if (da.logits != nullptr) da.stage_rows = keep_all_logits ? da.chunk : std::min(da.chunk, seg->max_vis_len);
    if (da.stage_rows > 3 * kLogitStageMaxRows) return ST3_ERR_UNSUPPORTED;    // 48 KB of LDS: a cache of more than 64 x 3 x 4096 rows
    da.pending = reinterpret_cast<int32_t*>(ws + wl.pending);
    da.k_new = k_new; da.v_new = v_new;
    da.out = out;
    da.defer = (want_mass && defer_mass) ? 1 : 0;
    const PlanStash ps = stash != nullptr ? *stash : PlanStash{};
    ST3_DISPATCH_KV(launch_attend, shape, kv, da, ps, B, st);
    const bool mass_now = want_mass && !defer_mass;
    // defer_merge: the caller's eviction plan merges the chunk partials (whole-step call)
    if ((da.nsplit > 1 && !defer_merge) || mass_now) {
        FinishArgs fa{};
        fa.part_o = da.part_o; fa.part_ml = da.part_ml; fa.logits = da.logits;
        fa.kv_len = seg->kv_len; fa.vis_len = seg->vis_len; fa.tail_start = seg->tail_start;
        fa.H = H; fa.nsplit = da.nsplit; fa.nsplit_cap = wl.nsplit_cap; fa.chunk = da.chunk;
        fa.capacity = kv->capacity; fa.max_vis = seg->max_vis_len; fa.max_kv = max_kv_len; fa.sys_len = seg->sys_len;
        fa.appended = k_new != nullptr ? 1 : 0;
        fa.out = (da.nsplit > 1 && !defer_merge) ? out : nullptr;
        fa.mass = mass_now ? vis_mass : nullptr; fa.mass_stride = mass_stride;
        ST3_DISPATCH(launch_finish, shape, fa, B, st);
    }
    return check_launch();
}

st3_status enqueue_append(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                          const void* k_new, const void* v_new, hipStream_t st) {
    const int B = shape->batch, H = shape->heads;
    AppendArgs aa{};
    aa.k = kv->k; aa.v = kv->v;
    aa.stride_b = kv->stride_b; aa.stride_h = kv->stride_h; aa.stride_t = kv->stride_t;
    aa.k_new = k_new; aa.v_new = v_new; aa.kv_len = seg->kv_len; aa.H = H; aa.capacity = kv->capacity;
    if (kv->format == ST3_KV_E4M3) { aa.k_scale = kv->k_scale; aa.v_scale = kv->v_scale; }
    ST3_DISPATCH_KV(launch_append, shape, kv, aa, B, seg->kv_len, st);
    return check_launch();
}

st3_status validate_kv(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg) {
    return check_kv(s, kv, seg);
}

st3_status validate_kv_value_only(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg) {
    return check_kv(s, kv, seg, true);
}

// Enqueues a lazy layer's attention (Eq. 6): the probabilities come from the attend launch that last
// used `src_workspace` (same batch, heads and lengths; cache capacity src_capacity), the values
// from `kv->v` plus - when v_new is given - the row being appended, which is stored on the way.
st3_status enqueue_inherit(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                           int32_t max_kv_len, const void* v_new, const void* src_workspace,
                           size_t src_workspace_bytes, int32_t src_capacity, void* out, void* workspace,
                           size_t workspace_bytes, hipStream_t st, const PlanStash* stash) {
    const int B = shape->batch, H = shape->heads, D = shape->head_dim;
    const DecodeWs wl = decode_ws(B, H, D, kv->capacity);
    const DecodeWs sl = decode_ws(B, H, D, src_capacity);
    if (workspace_bytes < wl.total || src_workspace_bytes < sl.total) return ST3_ERR_WORKSPACE_TOO_SMALL;
    if (max_kv_len > src_capacity) return ST3_ERR_INVALID_ARG;       // the source kept a logit per cached key
    char* ws = reinterpret_cast<char*>(workspace);
    const char* sws = reinterpret_cast<const char*>(src_workspace);
    InheritArgs ia{};
    ia.v = kv->v; ia.stride_b = kv->stride_b; ia.stride_h = kv->stride_h; ia.stride_t = kv->stride_t;
    ia.kv_len = seg->kv_len; ia.vis_len = seg->vis_len; ia.tail_start = seg->tail_start;
    ia.sys_len = seg->sys_len; ia.max_vis = seg->max_vis_len;
    ia.B = B; ia.max_kv = max_kv_len; ia.H = H;
    ia.nsplit = decode_nsplit(B, H, max_kv_len);
    if (ia.nsplit > wl.nsplit_cap) ia.nsplit = wl.nsplit_cap;
    ia.nsplit_cap = wl.nsplit_cap;
    ia.chunk = decode_chunk(max_kv_len, ia.nsplit);
    ia.nsplit = (max_kv_len + ia.chunk - 1) / ia.chunk;
    if (ia.nsplit < 1) ia.nsplit = 1;
    ia.src_logits = reinterpret_cast<const float*>(sws + sl.logits);
    ia.src_part_ml = reinterpret_cast<const float*>(sws + sl.part_ml);
    ia.src_pending = reinterpret_cast<const int32_t*>(sws + sl.pending);
    ia.src_capacity = src_capacity; ia.src_nsplit_cap = sl.nsplit_cap;
    ia.part_o = reinterpret_cast<float*>(ws + wl.part_o);
    ia.v_new = v_new; ia.out = out;
    if (kv->format == ST3_KV_E4M3) ia.v_scale = kv->v_scale;
    const PlanStash ps = stash != nullptr ? *stash : PlanStash{};
    ST3_DISPATCH_KV(launch_inherit, shape, kv, ia, ps, B, st);
    if (ia.nsplit > 1) {
        FinishArgs fa{};
        fa.part_o = ia.part_o; fa.kv_len = seg->kv_len; fa.vis_len = seg->vis_len; fa.tail_start = seg->tail_start;
        fa.sys_len = seg->sys_len; fa.max_vis = seg->max_vis_len;
        fa.H = H; fa.nsplit = ia.nsplit; fa.nsplit_cap = wl.nsplit_cap; fa.chunk = ia.chunk;
        fa.capacity = kv->capacity; fa.max_kv = max_kv_len; fa.plain_sum = 1;
        fa.appended = v_new != nullptr ? 1 : 0;
        fa.out = out;
        ST3_DISPATCH(launch_finish, shape, fa, B, st);
    }
    return check_launch();
}

}  // namespace st3

extern "C" st3_status st3_decode_attention(const st3_attn_shape* shape, const void* q, const st3_kv_layer* kv,
                                           const st3_segments* seg, void* out, float* vis_mass, int64_t mass_stride,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    st3_status s = st3::check_shape(shape);
    if (s != ST3_OK) return s;
    s = st3::validate_kv(shape, kv, seg);
    if (s != ST3_OK) return s;
    if (!q || !out || !workspace) return ST3_ERR_INVALID_ARG;
    if (!st3::aligned16(q) || !st3::aligned16(workspace)) return ST3_ERR_INVALID_ARG;
    if (vis_mass && mass_stride < seg->max_vis_len) return ST3_ERR_INVALID_ARG;
    return st3::enqueue_decode(shape, q, kv, seg, seg->max_kv_len, nullptr, nullptr, out, vis_mass, mass_stride,
                               vis_mass != nullptr, false, true, workspace, workspace_bytes,
                               reinterpret_cast<hipStream_t>(stream), false, nullptr);
}

extern "C" st3_status st3_decode_attention_inherit(const st3_attn_shape* shape, const st3_kv_layer* kv,
                                                   const st3_segments* seg, const void* src_workspace,
                                                   size_t src_workspace_bytes, int32_t src_kv_capacity, void* out,
                                                   void* workspace, size_t workspace_bytes, void* stream) {
    st3_status s = st3::check_shape(shape);
    if (s != ST3_OK) return s;
    s = st3::validate_kv_value_only(shape, kv, seg);
    if (s != ST3_OK) return s;
    if (!out || !workspace || !src_workspace || src_kv_capacity <= 0) return ST3_ERR_INVALID_ARG;
    if (!st3::aligned16(workspace) || !st3::aligned16(src_workspace)) return ST3_ERR_INVALID_ARG;
    return st3::enqueue_inherit(shape, kv, seg, seg->max_kv_len, nullptr, src_workspace, src_workspace_bytes,
                                src_kv_capacity, out, workspace, workspace_bytes,
                                reinterpret_cast<hipStream_t>(stream), nullptr);
}

extern "C" st3_status st3_quantize_rows(const st3_attn_shape* shape, const st3_tensor4* src, const st3_kv_layer* kv,
                                        int32_t which, int32_t n, void* stream) {
    using namespace st3;
    st3_status s = check_shape(shape);
    if (s != ST3_OK) return s;
    if (!src || !src->data || !kv || (which != 0 && which != 1) || n < 0) return ST3_ERR_INVALID_ARG;
    if (kv->format != ST3_KV_PLAIN && kv->format != ST3_KV_E4M3) return ST3_ERR_INVALID_ARG;
    if (kv->format == ST3_KV_E4M3 && shape->dtype != ST3_BF16) return ST3_ERR_UNSUPPORTED;
    void* dst = which == 0 ? kv->k : kv->v;
    const float* scale = kv->format == ST3_KV_E4M3 ? (which == 0 ? kv->k_scale : kv->v_scale) : nullptr;
    if (!dst || (kv->format == ST3_KV_E4M3 && !scale) || n > kv->capacity) return ST3_ERR_INVALID_ARG;
    const int eb = elem_bytes(shape->dtype), ceb = kv_elem_bytes(shape, kv);
    if (!aligned16(src->data) || !aligned16(dst)) return ST3_ERR_INVALID_ARG;
    if ((src->stride_t * eb) % 16 || (src->stride_h * eb) % 16 || (src->stride_b * eb) % 16) return ST3_ERR_INVALID_ARG;
    if ((kv->stride_t * ceb) % 16 || (kv->stride_h * ceb) % 16 || (kv->stride_b * ceb) % 16) return ST3_ERR_INVALID_ARG;
    if (src->stride_t < shape->head_dim || kv->stride_t < shape->head_dim) return ST3_ERR_INVALID_ARG;
    if (n == 0) return ST3_OK;
    QuantArgs qa{};
    qa.src = src->data; qa.s_sb = src->stride_b; qa.s_sh = src->stride_h; qa.s_st = src->stride_t;
    qa.dst = dst; qa.d_sb = kv->stride_b; qa.d_sh = kv->stride_h; qa.d_st = kv->stride_t;
    qa.scale = scale; qa.H = shape->heads; qa.n = n;
    ST3_DISPATCH_KV(launch_quantize, shape, kv, qa, shape->batch, reinterpret_cast<hipStream_t>(stream));
    return check_launch();
}

extern "C" st3_status st3_kv_append(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                                    const void* k_new, const void* v_new, void* stream) {
    st3_status s = st3::check_shape(shape);
    if (s != ST3_OK) return s;
    // a layer that caches V only (lazy layer of Alg. 2) passes kv->k == NULL and k_new == NULL
    const bool value_only = kv && !kv->k && !k_new;
    s = value_only ? st3::validate_kv_value_only(shape, kv, seg) : st3::validate_kv(shape, kv, seg);
    if (s != ST3_OK) return s;
    if ((!value_only && (!k_new || !st3::aligned16(k_new))) || !v_new || !st3::aligned16(v_new))
        return ST3_ERR_INVALID_ARG;
    if (seg->max_kv_len >= kv->capacity) return ST3_ERR_INVALID_ARG;
    return st3::enqueue_append(shape, kv, seg, k_new, v_new, reinterpret_cast<hipStream_t>(stream));
}
