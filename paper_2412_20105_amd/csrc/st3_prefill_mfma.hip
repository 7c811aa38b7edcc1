// bf16 prefill attention (Eq. 2, causal) on the MFMA units of gfx950, with the logits of the last
// W query rows saved for the visual mass (Sec. 3.2).
//
// Tiling.  A workgroup of 4 wavefronts owns 128 consecutive query rows (32 per wave) of one (b,h)
// and walks the key tiles of 64 keys up to its diagonal.  K and V tiles are staged in LDS once
// per workgroup; V is stored transposed (Vt[d][key]) because both MFMA operands want the
// contraction index contiguous per lane.
//
// Per wave and key tile, with v_mfma_f32_32x32x16_bf16 (A: 32 x 16, B: 16 x 32, C: 32 x 32; lane l
// holds A[l%32][8*(l/32)..+8], B[8*(l/32)..+8][l%32] and C[8*(r/4) + 4*(l/32) + r%4][l%32], r < 16):
//   S^T = K Q^T   A = K rows from LDS, B = Q fragments kept in registers.  A lane then owns ONE
//                 query (column l%32) and 16 of the 32 keys of a sub-tile, so the softmax row
//                 reductions are in-lane plus one exchange with lane l^32.
//   O^T = V^T P^T A = Vt rows from LDS, B = P^T taken straight from the S^T accumulator registers.
//                 The accumulator's row pattern fixes which keys a lane holds, so the contraction
//                 slots are assigned to keys in that pattern and Vt is read in the same pattern.
// Online softmax in the log2 domain, fp32.  For the second MFMA P is split into two bf16 terms,
// P = P_hi + P_lo (16 mantissa bits together), and both are multiplied by V: rounding P to one
// bf16 would put an error of 2^-9 of the row's magnitude on every output element, which is far
// above the element-wise tolerance for outputs that happen to be small.
#include "st3_prefill.h"

namespace st3 {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 128;            // queries per workgroup
constexpr int kBN = 64;             // keys per tile
constexpr int kVPad = kBN + 2;      // Vt row stride in elements: 33 words, so column reads spread over banks

union Frag {
    bf16x8 v;
    u32x4 u4;
    uint32_t w[4];
};

template <int NK, int NV>
struct TileRegs {
    u32x4 k[NK], va[NV], vb[NV];
};

// Issues the global loads of the K/V tile that starts at key k0 (rows past n-1 are clamped).
template <int D, int NK, int NV>
__device__ __forceinline__ void fetch_tile(TileRegs<NK, NV>& t, const uint16_t* Kp, const uint16_t* Vp, int64_t k_st,
                                           int64_t v_st, int k0, int n, int tid) {
    constexpr int VPR = D / 8;
#pragma unroll
    for (int i = 0; i < NK; ++i) {
        const int vec = tid + 256 * i;
        const int key = min(k0 + vec / VPR, n - 1);
        t.k[i] = *reinterpret_cast<const u32x4*>(Kp + (int64_t)key * k_st + (vec % VPR) * 8);
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int item = tid + 256 * i;
        const int cv = item % VPR, kp = item / VPR;
        const int key_a = min(k0 + 2 * kp, n - 1), key_b = min(k0 + 2 * kp + 1, n - 1);
        t.va[i] = *reinterpret_cast<const u32x4*>(Vp + (int64_t)key_a * v_st + cv * 8);
        t.vb[i] = *reinterpret_cast<const u32x4*>(Vp + (int64_t)key_b * v_st + cv * 8);
    }
}

__device__ __forceinline__ void put_pair(uint16_t* Vt, int col, int kp, uint32_t wa, uint32_t wb) {
    *reinterpret_cast<uint32_t*>(&Vt[col * kVPad + 2 * kp]) = (wa & 0xffffu) | (wb << 16);              // (key_a, key_b)
    *reinterpret_cast<uint32_t*>(&Vt[(col + 1) * kVPad + 2 * kp]) = (wa >> 16) | (wb & 0xffff0000u);
}

// Writes the staged tile to LDS: K row-major (padded), V transposed (a thread holds 2 adjacent
// keys x 8 columns and writes 8 words, one per column).
template <int D, int NK, int NV>
__device__ __forceinline__ void stage_tile(const TileRegs<NK, NV>& t, uint16_t* Ks, uint16_t* Vt, int tid) {
    constexpr int VPR = D / 8, KPAD = D + 8;
#pragma unroll
    for (int i = 0; i < NK; ++i) {
        const int vec = tid + 256 * i;
        *reinterpret_cast<u32x4*>(&Ks[(vec / VPR) * KPAD + (vec % VPR) * 8]) = t.k[i];
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int item = tid + 256 * i;
        const int cv = item % VPR, kp = item / VPR;
        put_pair(Vt, cv * 8 + 0, kp, t.va[i].x, t.vb[i].x);
        put_pair(Vt, cv * 8 + 2, kp, t.va[i].y, t.vb[i].y);
        put_pair(Vt, cv * 8 + 4, kp, t.va[i].z, t.vb[i].z);
        put_pair(Vt, cv * 8 + 6, kp, t.va[i].w, t.vb[i].w);
    }
}

// One-dimensional grid of ceil(n/128) * H * B workgroups (the mapping to query tile and strip is in the kernel).
// Register budget: two waves per SIMD (256 registers each), so that one wave's softmax VALU work
// overlaps the other's MFMAs.  The 64-key LDS tile is consumed as two 32-key halves, each with its
// own online-softmax update, which halves the live S/P registers; the accumulator is only rescaled
// when some row's maximum actually moved.  The next tile's global loads are issued before the
// current tile is consumed and written to LDS after it.
template <int D>
__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(PrefillArgs a) {
    constexpr int KS = D / 16;          // contraction steps of S^T
    constexpr int DT = D / 32;          // 32-row tiles of O^T
    constexpr int KPAD = D + 8;         // K row stride in LDS (elements)
    constexpr int VPR = D / 8;          // 16-byte vectors per row
    constexpr int KV_K = kBN * VPR / 256;           // K vectors staged per thread and tile
    constexpr int KV_V = (kBN / 2) * VPR / 256;     // V key-pair items per thread and tile
    __shared__ __attribute__((aligned(16))) uint16_t Ks[kBN * KPAD];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[D * kVPad];

    // Workgroup -> (query tile, strip).  Workgroups go round-robin by linear id to the 8 XCDs (checked
    // with a probe: XCC id == id % 8) and, within an XCD, in turn to its 4 shader engines; each XCD
    // has an L2 of its own; a causal query tile costs in proportion to its index.  With the query
    // tile as the fastest index, a tile count of 2 or 4 hands all heavy tiles to the same engines
    // (measured: 4 tiles per strip ran slower than 5).  So each of the 32 dispatch lanes
    // (id % 32) owns the strips congruent to it and receives the tiles of one strip back to back,
    // heaviest first: all lanes see the same cost sequence and a strip's K and V stay in one L2.
#ifndef ST3_PREFILL_LANES
#define ST3_PREFILL_LANES 32
#endif
    constexpr int kLanes = ST3_PREFILL_LANES;
    const int n_qt = a.n_qt, strips = a.H * a.B;
    const int full = strips / kLanes * kLanes;
    const int lin = blockIdx.x;
    int strip, qt;
    if (lin < full * n_qt) {
        const int dl = lin % kLanes, m = lin / kLanes;
        strip = (m / n_qt) * kLanes + dl;
        qt = n_qt - 1 - m % n_qt;
    } else {                                    // the strips left over when H*B is no multiple of 32
        const int r = lin - full * n_qt;
        strip = full + r / n_qt;
        qt = n_qt - 1 - r % n_qt;
    }
    const int h = strip % a.H, b = strip / a.H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, c = lane & 31;
    const int n = a.n;
    const int q0 = qt * kBM + wave * 32;
    const int myq = q0 + c;
    const int64_t bh = (int64_t)b * a.H + h;

    const uint16_t* Qp = reinterpret_cast<const uint16_t*>(a.q) + b * a.q_sb + h * a.q_sh;
    const uint16_t* Kp = reinterpret_cast<const uint16_t*>(a.k) + b * a.k_sb + h * a.k_sh;
    const uint16_t* Vp = reinterpret_cast<const uint16_t*>(a.v) + b * a.v_sb + h * a.v_sh;

    Frag qf[KS];
    {
        const uint16_t* qrow = Qp + (int64_t)min(myq, n - 1) * a.q_st;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s].u4 = *reinterpret_cast<const u32x4*>(qrow + 16 * s + 8 * g);
    }
    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    float m_i = -INFINITY, l_i = 0.f;

    // window rows (the last W queries) held by this wave?
    const bool wave_has_window = a.pre_logits != nullptr && q0 + 31 >= n - a.window && q0 < n;
    const int w_idx = myq - (n - a.window);
    const bool lane_in_window = wave_has_window && w_idx >= 0 && myq < n;
    float* lg_row = lane_in_window ? a.pre_logits + (bh * a.window + w_idx) * a.vis_len : nullptr;

    // global -> register staging of one K/V tile (rows past the end are clamped and masked later)
    TileRegs<KV_K, KV_V> tr;
    const int k_end = min(n, qt * kBM + kBM);           // keys this workgroup can see
    fetch_tile<D>(tr, Kp, Vp, a.k_st, a.v_st, 0, n, tid);
    for (int k0 = 0; k0 < k_end; k0 += kBN) {
        __syncthreads();                                // previous tile fully consumed
        stage_tile<D>(tr, Ks, Vt, tid);
        __syncthreads();
        if (k0 + kBN < k_end) fetch_tile<D>(tr, Kp, Vp, a.k_st, a.v_st, k0 + kBN, n, tid);   // in flight while this tile is consumed
        if (k0 > q0 + 31 || q0 >= n) continue;          // tile entirely above this wave's diagonal, or a wave whose
                                                        // 32 queries all lie beyond the prompt (ragged last tile)

#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int ks0 = k0 + 32 * sub;
            if (ks0 > q0 + 31) break;                   // this half is above the diagonal too
            // ---- S^T = K Q^T for 32 keys ------------------------------------------------------
            f32x16 sacc;
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                Frag ka;
                ka.u4 = *reinterpret_cast<const u32x4*>(&Ks[(32 * sub + c) * KPAD + 16 * s + 8 * g]);
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.v, qf[s].v, sacc, 0, 0, 0);
            }
            // ---- scale, causal / length mask, row maximum -----------------------------------
            float mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = ks0 + 8 * (r / 4) + 4 * g + (r % 4);
                float s = sacc[r] * a.scale_l2;
                if (key > myq || key >= n) s = -INFINITY;
                sacc[r] = s;
                mx = fmaxf(mx, s);
            }
            if (wave_has_window && lg_row != nullptr) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = ks0 + 8 * (r / 4) + 4 * g + (r % 4);
                    if (key >= a.sys_len && key < a.sys_len + a.vis_len && key <= myq) lg_row[key - a.sys_len] = sacc[r];
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // The first half of a tile always holds a visible key for every row (k0 <= q0 <= myq);
            // the second half may be entirely masked for some rows, then mx = -inf and m stays.
            const float m_new = fmaxf(m_i, mx);
            const bool moved = m_new > m_i;
            const float alpha = exp2_fast(m_i - m_new);     // m_i = -inf only before the first key: alpha = 0
            m_i = m_new;
            float psum = 0.f;
            Frag pb[2], pl[2];
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float p = exp2_fast(sacc[8 * kk + j] - m_new);
                    psum += p;
                    const __bf16 hi = (__bf16)p;
                    pb[kk].v[j] = hi;
                    pl[kk].v[j] = (__bf16)(p - (float)hi);
                }
            l_i = l_i * alpha + psum;
            if (__any(moved)) {                         // rescale only when some row's maximum moved
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
            }
            // ---- O^T += V^T P^T ---------------------------------------------------------------
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int base = 32 * sub + 16 * kk + 4 * g;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const uint16_t* row = &Vt[(32 * dt + c) * kVPad + base];
                    Frag va;
                    va.w[0] = *reinterpret_cast<const uint32_t*>(row);
                    va.w[1] = *reinterpret_cast<const uint32_t*>(row + 2);
                    va.w[2] = *reinterpret_cast<const uint32_t*>(row + 8);
                    va.w[3] = *reinterpret_cast<const uint32_t*>(row + 10);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.v, pb[kk].v, oacc[dt], 0, 0, 0);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.v, pl[kk].v, oacc[dt], 0, 0, 0);
                }
            }
        }
    }
    // ---- normalise and store -----------------------------------------------------------------
    const float l_tot = l_i + __shfl_xor(l_i, 32);
    const float rl = 1.0f / l_tot;
    if (myq < n) {
        uint16_t* orow = reinterpret_cast<uint16_t*>(a.out) + b * a.o_sb + h * a.o_sh + (int64_t)myq * a.o_st;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int dd = 32 * dt + 8 * rq + 4 * g;
                uint2 pk;
                pk.x = f32_to_bf16_bits(oacc[dt][4 * rq] * rl) | (f32_to_bf16_bits(oacc[dt][4 * rq + 1] * rl) << 16);
                pk.y = f32_to_bf16_bits(oacc[dt][4 * rq + 2] * rl) | (f32_to_bf16_bits(oacc[dt][4 * rq + 3] * rl) << 16);
                *reinterpret_cast<uint2*>(orow + dd) = pk;
            }
        if (lane_in_window && g == 0) {
            a.pre_ml[(bh * a.window + w_idx) * 2] = m_i;
            a.pre_ml[(bh * a.window + w_idx) * 2 + 1] = l_tot;
        }
    }
}

}  // namespace

st3_status launch_prefill_mfma(const PrefillArgs& a, int B, int D, hipStream_t st) {
    // 8-byte output stores and 16-byte input loads need these alignments (rows are 16-byte aligned already)
    PrefillArgs pa = a;
    pa.n_qt = (a.n + kBM - 1) / kBM;
    pa.B = B;
    const int64_t wgs = (int64_t)pa.n_qt * a.H * B;
    if (wgs > 0x7fffffff) return ST3_ERR_UNSUPPORTED;
    dim3 grid((unsigned)wgs);
    if (D == 128) prefill_mfma_kernel<128><<<grid, 256, 0, st>>>(pa);
    else if (D == 64) prefill_mfma_kernel<64><<<grid, 256, 0, st>>>(pa);
    else return ST3_ERR_UNSUPPORTED;
    return ST3_OK;
}

}  // namespace st3
