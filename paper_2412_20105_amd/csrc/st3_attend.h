// One wavefront streaming a range of cached K/V rows for a single query (Eq. 2 with one row).
//
// Layout of the work inside the wave: a row of D elements is 16*LPR bytes, so LPR consecutive
// lanes each own a 16-byte slice of it and one 64-lane load instruction fetches RPL = 64/LPR
// whole rows, fully coalesced.  Lane l therefore always sees row-group l / LPR and column slice
// l % LPR, for K and for V alike: the logit of a row is reduced over the LPR lanes that hold it
// (DPP), and the probability it yields multiplies exactly the V slice the same lane has loaded.
// U such loads of K and U of V are in flight per tile, i.e. U*RPL keys.
#pragma once

#include "st3_common.h"

namespace st3 {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 load16_nt(const void* p) {
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// NT = true: the data is read exactly once (decode streams K and V), so the load is marked
// non-temporal; measured +17 % bandwidth on the decode kernel.  NT = false where rows are re-read.
template <bool NT>
__device__ __forceinline__ uint4 load16(const void* p) {
    if (NT) return load16_nt(p);
    return *reinterpret_cast<const uint4*>(p);
}

template <typename T, int D>
struct RowMap {
    static constexpr int EPL = ElemTraits<T>::kPerVec;          // elements per lane
    static constexpr int LPR = D / EPL;                         // lanes per row
    static constexpr int RPL = kWave / LPR;                     // rows per wave-wide load
};

template <typename T, int D>
__device__ __forceinline__ void load_q_slice(const T* qrow, int lane, float* qf) {
    using M = RowMap<T, D>;
    uint4 raw = *reinterpret_cast<const uint4*>(qrow + (lane % M::LPR) * M::EPL);
    ElemTraits<T>::unpack(raw, qf);
}

// This lane's slice of a [d] row of elements T when the lane map is that of cache elements KT
// (RowMap<KT, D>::EPL elements per lane, which is more than one 16-byte vector of T when KT is
// narrower than T), as floats.
template <typename T, typename KT, int D>
__device__ __forceinline__ void load_row_slice(const T* row, int lane, float* f) {
    using M = RowMap<KT, D>;
    constexpr int PV = ElemTraits<T>::kPerVec, NV = M::EPL / PV;
    static_assert(M::EPL % PV == 0, "a lane's slice is a whole number of 16-byte vectors");
    const T* p = row + (lane % M::LPR) * M::EPL;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint4 raw = *reinterpret_cast<const uint4*>(p + i * PV);
        ElemTraits<T>::unpack(raw, f + i * PV);
    }
}

// Online-softmax state of one wave.  `l` holds, per lane, the sum of probabilities over the rows
// of that lane's row-group only; `acc` likewise.  finish_wave() folds the row-groups together.
template <int EPL>
struct WaveState {
    float m;            // running maximum (log2 domain), wave-uniform
    float l;
    float acc[EPL];
};

// Streams the tiles of U*RPL rows that start at r0, r0+step, r0+2*step, ... below r1; within a
// tile only rows < r1 count.  `safe_row` is any row of the strip that may be read (lanes whose
// row falls outside load it instead and are masked).  kbase/vbase point at row 0 of the (b,h)
// strip.  logit_out (may be null): float array indexed by (row - vis_lo) for rows in
// [vis_lo, vis_hi), receives the scaled logit in the log2 domain.
template <typename T, int D, int U, bool NT>
__device__ __forceinline__ void wave_attend(const float* qf, const T* kbase, const T* vbase, int64_t stride_t,
                                            int r0, int r1, int step, int safe_row, float scale_l2, int lane,
                                            WaveState<RowMap<T, D>::EPL>& st,
                                            float* logit_out, int vis_lo, int vis_hi) {
    using M = RowMap<T, D>;
    constexpr int EPL = M::EPL, LPR = M::LPR, RPL = M::RPL;
    const int grp = lane / LPR;
    const int64_t col = (int64_t)(lane % LPR) * EPL;
    for (int t0 = r0; t0 < r1; t0 += step) {
        uint4 kr[U], vr[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int row = t0 + u * RPL + grp;
            ok[u] = row < r1;
            int64_t off = (int64_t)(ok[u] ? row : safe_row) * stride_t + col;
            kr[u] = load16<NT>(kbase + off);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int row = t0 + u * RPL + grp;
            int64_t off = (int64_t)(ok[u] ? row : safe_row) * stride_t + col;
            vr[u] = load16<NT>(vbase + off);
        }
        float s[U];
        float mt = -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[EPL];
            ElemTraits<T>::unpack(kr[u], kf);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) part = fmaf(qf[e], kf[e], part);
            part = group_sum<LPR>(part) * scale_l2;
            int row = t0 + u * RPL + grp;
            if (logit_out != nullptr && ok[u] && (lane % LPR) == 0 && row >= vis_lo && row < vis_hi)
                logit_out[row - vis_lo] = part;
            s[u] = ok[u] ? part : -INFINITY;
            mt = fmaxf(mt, s[u]);
        }
        mt = wave_max_from<LPR>(mt);
        float m_new = fmaxf(st.m, mt);
        float alpha = exp2_fast(st.m - m_new);       // first tile: exp2(-inf) = 0
        st.m = m_new;
        st.l *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) st.acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float p = exp2_fast(s[u] - m_new);       // masked rows: exp2(-inf) = 0
            st.l += p;
            float vf[EPL];
            ElemTraits<T>::unpack(vr[u], vf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) st.acc[e] = fmaf(p, vf[e], st.acc[e]);
        }
    }
}

// Where the rows a wave walks over sit in the strip.  A cache may keep its never-pruned tail
// (instruction and generated rows) at a fixed row offset while the visual segment in front of it
// shrinks: the rows the attention sees are then numbered without the gap, and row r of that
// numbering is stored at r (r < split_row) or at r + gap.  {INT_MAX, 0}: no gap.
struct RowShift {
    int split_row;
    int gap;
    __device__ __forceinline__ int physical(int r) const { return r + (r >= split_row ? gap : 0); }
};

// The two layouts of the rows behind the visual segment, resolved for one sequence: `len_phys`
// rows exist physically; tail_start == null: they are contiguous; else the tail begins at
// tail_start[b] and the rows between the visual segment and it are dead.
struct SeqLayout {
    int nv;         // visual rows
    int base;       // sys_len + nv: first row behind the visual segment in the gap-free numbering
    int gap;        // dead rows between the segment and the tail
    int vlen;       // rows the attention sees
    __device__ __forceinline__ RowShift shift() const { return RowShift{base, gap}; }
};
__device__ __forceinline__ SeqLayout seq_layout(int sys_len, int vis_len_b, int max_vis, int len_phys,
                                                const int32_t* tail_start, int b) {
    SeqLayout L;
    L.nv = max(0, min(vis_len_b, max_vis));
    L.base = min(sys_len + L.nv, max(len_phys, 0));
    const int ts = tail_start ? tail_start[b] : L.base;
    L.gap = ts > L.base ? ts - L.base : 0;
    L.vlen = L.base + max(0, len_phys - (L.base + L.gap));
    return L;
}

// Issues the loads of the tile of U*RPL rows that starts at t0: rows >= bound read `safe_row` instead.
template <typename T, int D, int U, bool NT>
__device__ __forceinline__ void issue_tile(const T* kbase, const T* vbase, int64_t stride_t, int t0, int bound,
                                           int safe_row, int lane, uint4 (&k)[U], uint4 (&v)[U],
                                           const RowShift sh = RowShift{0x7fffffff, 0}) {
    using M = RowMap<T, D>;
    const int grp = lane / M::LPR;
    const int64_t col = (int64_t)(lane % M::LPR) * M::EPL;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int row = t0 + u * M::RPL + grp;
        k[u] = load16<NT>(kbase + (int64_t)sh.physical(row < bound ? row : safe_row) * stride_t + col);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int row = t0 + u * M::RPL + grp;
        v[u] = load16<NT>(vbase + (int64_t)sh.physical(row < bound ? row : safe_row) * stride_t + col);
    }
}

// The same for a tile whose placement is a guess (`sh` may be wrong for this sequence): rows of the
// tile at or beyond row_bound, and rows that `sh` would place at or beyond phys_bound, read
// `safe_row` (< row_bound, taken as stored where it is numbered) instead, so every address stays
// below phys_bound whatever the guess.
template <typename T, int D, int U, bool NT>
__device__ __forceinline__ void issue_tile_within(const T* kbase, const T* vbase, int64_t stride_t, int t0, int row_bound,
                                                  int phys_bound, int safe_row, int lane, uint4 (&k)[U], uint4 (&v)[U],
                                                  const RowShift sh) {
    using M = RowMap<T, D>;
    const int grp = lane / M::LPR;
    const int64_t col = (int64_t)(lane % M::LPR) * M::EPL;
    int64_t off[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int row = t0 + u * M::RPL + grp;
        const int p = sh.physical(row);
        off[u] = (int64_t)((row < row_bound && p < phys_bound) ? p : safe_row) * stride_t + col;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) k[u] = load16<NT>(kbase + off[u]);
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = load16<NT>(vbase + off[u]);
}

// Same contract as wave_attend, software-pipelined: the loads of tile i+1 are issued before tile i
// is consumed, so a wave always has 2*U loads in flight while it computes.  The loads of the first
// tile (rows from r0) have been issued by the caller into kr/vr with issue_tile(); any bound >= r1
// that keeps the reads inside the strip will do there, which lets a kernel issue them before it
// knows the sequence length.
template <typename T, int D, int U, bool NT>
__device__ __forceinline__ void wave_attend_primed(const float* qf, const T* kbase, const T* vbase, int64_t stride_t,
                                                   int r0, int r1, int step, int safe_row, float scale_l2, int lane,
                                                   WaveState<RowMap<T, D>::EPL>& st, float* logit_out, int vis_lo,
                                                   int vis_hi, uint4 (&kr)[U], uint4 (&vr)[U],
                                                   const RowShift sh = RowShift{0x7fffffff, 0}) {
    using M = RowMap<T, D>;
    constexpr int EPL = M::EPL, LPR = M::LPR, RPL = M::RPL;
    const int grp = lane / LPR;
    if (r0 >= r1) return;
    uint4 kn[U], vn[U];
    for (int t0 = r0; t0 < r1; t0 += step) {
        const int tn = t0 + step;
        if (tn < r1) issue_tile<T, D, U, NT>(kbase, vbase, stride_t, tn, r1, safe_row, lane, kn, vn, sh);
        float s[U];
        float mt = -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[EPL];
            ElemTraits<T>::unpack(kr[u], kf);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) part = fmaf(qf[e], kf[e], part);
            part = group_sum<LPR>(part) * scale_l2;
            int row = t0 + u * RPL + grp;
            const bool ok = row < r1;
            if (logit_out != nullptr && ok && (lane % LPR) == 0 && row >= vis_lo && row < vis_hi)
                logit_out[row - vis_lo] = part;
            s[u] = ok ? part : -INFINITY;
            mt = fmaxf(mt, s[u]);
        }
        mt = wave_max_from<LPR>(mt);
        float m_new = fmaxf(st.m, mt);
        float alpha = exp2_fast(st.m - m_new);
        st.m = m_new;
        st.l *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) st.acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float p = exp2_fast(s[u] - m_new);
            st.l += p;
            float vf[EPL];
            ElemTraits<T>::unpack(vr[u], vf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) st.acc[e] = fmaf(p, vf[e], st.acc[e]);
        }
        if (tn < r1) {
#pragma unroll
            for (int u = 0; u < U; ++u) { kr[u] = kn[u]; vr[u] = vn[u]; }
        }
    }
}

// One more row for a wave's state, from registers: kraw/vraw hold this lane's 16-byte slices of the
// row (every row-group holds the same row; only group 0 counts it).
template <typename T, int D>
__device__ __forceinline__ void wave_attend_row(const float* qf, uint4 kraw, uint4 vraw, int row, float scale_l2,
                                                int lane, WaveState<RowMap<T, D>::EPL>& st, float* logit_out,
                                                int vis_lo, int vis_hi) {
    using M = RowMap<T, D>;
    constexpr int EPL = M::EPL, LPR = M::LPR;
    float kf[EPL], vf[EPL];
    ElemTraits<T>::unpack(kraw, kf);
    ElemTraits<T>::unpack(vraw, vf);
    float part = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) part = fmaf(qf[e], kf[e], part);
    part = group_sum<LPR>(part) * scale_l2;
    if (logit_out != nullptr && lane == 0 && row >= vis_lo && row < vis_hi) logit_out[row - vis_lo] = part;
    const float m_new = fmaxf(st.m, part);
    const float alpha = exp2_fast(st.m - m_new);
    st.m = m_new;
    st.l *= alpha;
    const float p = lane < LPR ? exp2_fast(part - m_new) : 0.f;
    st.l += p;
#pragma unroll
    for (int e = 0; e < EPL; ++e) st.acc[e] = fmaf(p, vf[e], st.acc[e] * alpha);
}

// Folds the row-groups of a wave together: afterwards every lane holds the wave's total l and
// the total acc for its column slice.
template <typename T, int D>
__device__ __forceinline__ void finish_wave(WaveState<RowMap<T, D>::EPL>& st) {
    using M = RowMap<T, D>;
    st.l = wave_sum_from<M::LPR>(st.l);
#pragma unroll
    for (int e = 0; e < M::EPL; ++e) st.acc[e] = wave_sum_from<M::LPR>(st.acc[e]);
}

}  // namespace st3
