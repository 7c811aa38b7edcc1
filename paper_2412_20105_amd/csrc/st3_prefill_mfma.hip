// bf16 prefill attention (Eq. 2, causal) on the MFMA units of gfx950, with the logits of the last
// W query rows saved for the visual mass (Sec. 3.2).
//
// Tiling.  A workgroup of 4 wavefronts owns 128 consecutive query rows (32 per wave) of one (b,h)
// and walks the key tiles of 64 keys up to its diagonal.  K and V tiles live in LDS, row-major, in
// two buffers.  They get there by direct global-to-LDS loads (no staging registers; a strip's base
// address in scalar registers, 32 bits of offset per lane): the tile after the current one is in
// flight while the current one is consumed, and a tile costs one barrier.
// A direct load writes the 64 x 16 bytes of a wave to consecutive LDS addresses, so rows cannot be
// padded against bank conflicts; instead every lane chooses WHICH 16 bytes of its row it fetches,
// which stores the row's 16-byte units permuted (unit u of row r holds column unit u ^ swz(r)).
//
// Per wave, with v_mfma_f32_32x32x16_bf16 (A: 32 x 16, B: 16 x 32, C: 32 x 32; lane l holds
// A[l%32][8*(l/32)..+8], B[8*(l/32)..+8][l%32] and C[8*(r/4) + 4*(l/32) + r%4][l%32], r < 16):
//   S^T = K Q^T   A = K rows from LDS (one 16-byte read per lane), B = Q fragments kept in
//                 registers.  A lane then owns ONE query (column l%32) and 16 of the 32 keys of a
//                 sub-tile, so the softmax row reductions are in-lane plus one exchange with lane l^32.
//   O^T = V^T P^T B = P^T taken straight from the S^T accumulator registers, which fixes which keys
//                 sit in which contraction slot: slots 8g..8g+3 of the MFMA over keys 16kk..16kk+15
//                 are keys 16kk+4g..+3, slots 8g+4..8g+7 keys 16kk+8+4g..+3.  A = V^T in the same
//                 pattern: a lane needs, for ONE column d of V, two runs of four consecutive keys,
//                 which is what the LDS transpose read of gfx950 (ds_read_b64_tr_b16) returns from
//                 a row-major tile: within 16 lanes, lane i passes the address of elements
//                 4*(i%4)..+3 of row i/4 of a 4 x 16 block and receives column i of that block
//                 (layout checked on the device with an index pattern).
// A tile that lies entirely below a wave's diagonal is consumed whole (64 keys, one softmax
// update); on the diagonal the 32-key sub-tile that holds it is masked and a sub-tile above it is
// skipped.  Online softmax in the log2 domain, fp32; the softmax scale is folded into the
// exponent's multiply-add.  For the second MFMA P is split into two bf16 terms, P = P_hi + P_lo
// (P_hi the upper 16 bits of the float, P_lo the rounded rest: 16 mantissa bits together), and both
// are multiplied by V: rounding P to one bf16 would put an error of 2^-9 of the row's magnitude on
// every output element, far above the element-wise tolerance for outputs that happen to be small.
#include "st3_prefill.h"

namespace st3 {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 128;            // queries per workgroup
constexpr int kBN = 64;             // keys per tile

// An LDS tile is kBN rows of D elements, no padding.  The 64 banks are 256 bytes wide together, so
// RPB rows share one pass over the banks.  K rows are read 16 bytes per lane by lanes holding
// consecutive rows: unit u ^ ((r / RPB) % UPR) spreads 16 consecutive rows over all banks.  V rows
// are read by the transpose read, 32 lanes covering 4 consecutive rows x 64 bytes (4 units): the
// permutation 4 * ((r / RPB) % (UPR / 4)) puts the four rows on disjoint quarters of the banks.
template <int D> struct TileLayout {
    static constexpr int UPR = D / 8;                   // 16-byte units per row
    static constexpr int RPB = 256 / (2 * D);           // rows per 256 bytes: 1 or 2
    static constexpr int RPI = 1024 / (2 * D);          // rows per wave-wide direct load (1 KB): 4 or 8
    static constexpr int NI = kBN / (RPI * 4);          // direct loads of K, and of V, per wave and tile
    static constexpr int TILE = kBN * D;                // elements of one K (or V) tile
    __device__ static __forceinline__ int k_swz(int row) { return (row / RPB) & (UPR - 1); }
    __device__ static __forceinline__ int v_swz(int row) { return 4 * ((row / RPB) & (UPR / 4 - 1)); }
};

union Frag {
    bf16x8 v;
    u32x4 u4;
    uint32_t w[4];
    i16x4 h[2];
};

// One wave-wide direct load: every lane fetches the 16 bytes at base + lane_byte_off (global memory;
// the base is the same for all lanes and sits in scalar registers, the offset is 32 bits wide) and
// the wave's 64 x 16 bytes land at LDS byte address lds_byte_addr .. + 1023 in lane order (gfx950:
// global_load_lds_dwordx4, LDS base in M0).  Issued through inline assembly: the compiler treats the
// builtin form as an access that is outstanding on the LDS counter as well, and then makes every
// later wait for an LDS read a wait for ALL LDS reads in flight, which serialises the fragment
// reads of the whole tile.  What it does not know about is handled here: wait_direct_loads() before
// the barrier that publishes a buffer; M0 is declared clobbered; "memory" keeps LDS reads in place.
__device__ __forceinline__ void direct_load16(const uint16_t* base, uint32_t lane_byte_off, uint32_t lds_byte_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_byte_addr), "v"(lane_byte_off), "s"(base)
                 : "memory", "m0");
}

// A value that is the same in every lane, moved to scalar registers.
__device__ __forceinline__ const uint16_t* uniform_ptr(const uint16_t* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const uint16_t*>(((uint64_t)hi << 32) | lo);
}

// LDS byte address of a __shared__ object.
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const void*)p);
}

// Starts the direct loads of the K/V tile at key k0 into the buffer at LDS byte address `lds_buf` (K
// tile, then V tile).  Rows past n-1 are clamped: such keys lie above every valid query's diagonal
// and are masked there.  Every address read is a row of the caller's tensors; every LDS address
// written lies inside the buffer.
// Kp / Vp: row 0 of the strip (uniform).  k_lane / v_lane: byte offset of this lane's 16 bytes within
// the first 1 KB group of a tile at key 0 (row min(row0, n-1) and permuted unit folded in).
// Offsets from the strip's row 0 fit 32 bits (checked by the launcher).  wave_s: the wave's index, scalar.
template <int D>
__device__ __forceinline__ void issue_tile(uint32_t lds_buf, const uint16_t* Kp, const uint16_t* Vp, uint32_t k_lane,
                                           uint32_t v_lane, int64_t k_st, int64_t v_st, int k0, int n, int lane, int wave,
                                           int wave_s) {
    using L = TileLayout<D>;
    const int row0 = wave * L::RPI + lane / L::UPR;     // this lane's row in the wave's first group
    if (k0 + kBN <= n) {                                // all rows of the tile exist: plain strides
#pragma unroll
        for (int i = 0; i < L::NI; ++i) {
            const uint32_t dst = lds_buf + (4 * i + wave_s) * 1024;    // which 1 KB of the tile this wave-wide load fills
            const int key = k0 + 4 * i * L::RPI;
            direct_load16(uniform_ptr(Kp + key * k_st), k_lane, dst);
            direct_load16(uniform_ptr(Vp + key * v_st), v_lane, dst + 2 * L::TILE);
        }
    } else {
        const uint16_t* Ku = uniform_ptr(Kp);
        const uint16_t* Vu = uniform_ptr(Vp);
#pragma unroll
        for (int i = 0; i < L::NI; ++i) {
            const uint32_t dst = lds_buf + (4 * i + wave_s) * 1024;
            const int key = max(0, min(k0 + 4 * i * L::RPI, n - 1 - row0));     // this lane's row, key + row0, stays <= n - 1
            direct_load16(Ku, k_lane + (uint32_t)key * (uint32_t)(2 * k_st), dst);
            direct_load16(Vu, v_lane + (uint32_t)key * (uint32_t)(2 * v_st), dst + 2 * L::TILE);
        }
    }
}

// x of this lane and x of lane ^ 32 (v_permlane32_swap: lanes 32..63 of its first operand trade places
// with lanes 0..31 of its second; with both operands x, the one ends up holding the lower half's
// values in both halves and the other the upper half's).  No LDS round trip, unlike a shuffle.
__device__ __forceinline__ void both_halves(float x, float& a, float& b) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}

// All direct loads this wave has issued have landed in LDS (vmcnt(0); other counters untouched).
__device__ __forceinline__ void wait_direct_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// LDS transpose read: 4 consecutive rows of one column (see the header comment for the lane map).
__device__ __forceinline__ i16x4 lds_read_tr(const uint16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p));
}

// What a lane needs to find its operands in a tile (element offsets, fixed for the whole kernel).
template <int D>
struct LaneMap {
    int koff[D / 16];       // K fragment s of row c: row * D + ((2s + g) ^ k_swz) * 8
    int voff[D / 32];       // transpose read of d-tile dt: row (4g + (c%16)/4), unit (4dt + 2(c/16) + (c%4)/2) ^ v_swz, half c%2
    __device__ __forceinline__ void init(int c, int g) {
        using L = TileLayout<D>;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) koff[s] = c * D + ((2 * s + g) ^ L::k_swz(c)) * 8;
        const int row = 4 * g + ((c & 15) >> 2);
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
            voff[dt] = row * D + ((4 * dt + 2 * (c >> 4) + ((c & 3) >> 1)) ^ L::v_swz(row)) * 8 + 4 * (c & 1);
    }
};

// NSUB 32-key sub-tiles of the tile in (Kt, Vt) for one wave: S^T, one online-softmax update over
// all NSUB * 32 keys, O^T += V^T P^T.  DIAG: the last of them lies on the wave's diagonal (its keys
// start at the wave's first query), the only place where some keys are invisible to some rows.
template <int D, int NSUB, bool DIAG>
__device__ __forceinline__ void tile_step(const uint16_t* Kt, const uint16_t* Vt, const Frag* qf, f32x16* oacc,
                                          float& m_i, float& l_i, float scale_l2, const LaneMap<D>& lm, int c, int g,
                                          int k0, int myq, float* lg_row, int vis_lo, int vis_hi) {
    constexpr int KS = D / 16, DT = D / 32;
    // LDS reads are issued in batches ahead of their use, so that their latency is paid once per
    // batch and not once per MFMA: K fragments in groups of four contraction steps, the next group on
    // its way while the current one is multiplied.
    // ---- S^T = K Q^T ----------------------------------------------------------------------------
    constexpr int KG = 4, GPS = KS / KG, NG = NSUB * GPS;       // steps per group, groups per sub-tile, groups
    Frag ka[2][KG];
    f32x16 sacc[NSUB];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[sub][r] = 0.f;
#pragma unroll
    for (int s = 0; s < KG; ++s) ka[0][s].u4 = *reinterpret_cast<const u32x4*>(Kt + lm.koff[s]);
#pragma unroll
    for (int grp = 0; grp < NG; ++grp) {
        if (grp + 1 < NG) {
            const int sub = (grp + 1) / GPS, s0 = ((grp + 1) % GPS) * KG;
#pragma unroll
            for (int s = 0; s < KG; ++s)
                ka[(grp + 1) & 1][s].u4 = *reinterpret_cast<const u32x4*>(Kt + 32 * sub * D + lm.koff[s0 + s]);
        }
        __builtin_amdgcn_sched_barrier(0);
        const int sub = grp / GPS, s0 = (grp % GPS) * KG;
#pragma unroll
        for (int s = 0; s < KG; ++s)
            sacc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[grp & 1][s].v, qf[s0 + s].v, sacc[sub], 0, 0, 0);
    }
    Frag va[2][DT];                     // V^T fragments of the 16-key group in use and of the next one
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {   // the first group lands while the softmax runs
        va[0][dt].h[0] = lds_read_tr(Vt + lm.voff[dt]);
        va[0][dt].h[1] = lds_read_tr(Vt + 8 * D + lm.voff[dt]);
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- causal mask (diagonal sub-tile only), row maximum ----------------------------------------
    if (DIAG) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (8 * (r / 4) + 4 * g + (r % 4) > c) sacc[NSUB - 1][r] = -INFINITY;
    }
    if (lg_row != nullptr) {            // a row of the score window: keep the scaled logits of its visual keys
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = k0 + 32 * sub + 8 * (r / 4) + 4 * g + (r % 4);
                if (key >= vis_lo && key < vis_hi && key <= myq) lg_row[key - vis_lo] = sacc[sub][r] * scale_l2;
            }
    }
    float mx = sacc[0][0];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[sub][r]);
    {
        float lo_half, hi_half;
        both_halves(mx, lo_half, hi_half);
        mx = fmaxf(lo_half, hi_half);
    }
    // every row sees the first key of every tile it gets here (k0 <= q0 <= myq), so mx is finite.
    // The reference point m_i of the exponents only follows the row maximum when that has moved by
    // more than kLazy (probabilities then reach 2^kLazy at most, far inside fp32 and bf16 range):
    // a softmax is invariant to the reference point, and the accumulator rescaling it triggers
    // becomes rare instead of happening in nearly every tile.
    constexpr float kLazy = 8.0f;
    const float m_cand = fmaxf(m_i, mx * scale_l2);
    const bool moved = m_cand - m_i > kLazy;            // m_i = -inf before the first key: moved
    const float m_new = moved ? m_cand : m_i;
    const float alpha = exp2_fast(m_i - m_new);         // 1 when not moved; 0 before the first key
    m_i = m_new;
    float psum = 0.f;
    Frag pb[NSUB][2], pl[NSUB][2];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float p0 = exp2_fast(fmaf(sacc[sub][8 * kk + 2 * j], scale_l2, -m_new));      // masked: exp2(-inf) = 0
                const float p1 = exp2_fast(fmaf(sacc[sub][8 * kk + 2 * j + 1], scale_l2, -m_new));
                psum += p0 + p1;
                const uint32_t b0 = __float_as_uint(p0), b1 = __float_as_uint(p1);
                pb[sub][kk].w[j] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);      // upper halves of (p0, p1)
                const f32x2 lo = {p0 - __uint_as_float(b0 & 0xffff0000u), p1 - __uint_as_float(b1 & 0xffff0000u)};
                pl[sub][kk].w[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
            }
    l_i = l_i * alpha + psum;
    if (__any(moved)) {                                 // rescale only when some row's maximum moved
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
    }
    // ---- O^T += V^T P^T, 16 keys (one contraction) at a time ------------------------------------
#pragma unroll
    for (int grp = 0; grp < 2 * NSUB; ++grp) {
        if (grp + 1 < 2 * NSUB) {       // the next group's fragments are on their way while this one is used
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                va[(grp + 1) & 1][dt].h[0] = lds_read_tr(Vt + 16 * (grp + 1) * D + lm.voff[dt]);
                va[(grp + 1) & 1][dt].h[1] = lds_read_tr(Vt + (16 * (grp + 1) + 8) * D + lm.voff[dt]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[grp & 1][dt].v, pb[grp / 2][grp % 2].v, oacc[dt], 0, 0, 0);
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[grp & 1][dt].v, pl[grp / 2][grp % 2].v, oacc[dt], 0, 0, 0);
        }
    }
}

// The part of the tile at k0 that the wave with first query q0 can see (k0 <= q0).
template <int D>
__device__ __forceinline__ void consume_tile(const uint16_t* buf, int k0, int q0, const Frag* qf, f32x16* oacc,
                                             float& m_i, float& l_i, float scale_l2, const LaneMap<D>& lm, int c, int g,
                                             int myq, float* lg_row, int vis_lo, int vis_hi) {
    const uint16_t* Kt = buf;
    const uint16_t* Vt = buf + TileLayout<D>::TILE;
    if (k0 + kBN <= q0)         // below the diagonal: all 64 keys visible to all 32 rows
        tile_step<D, 2, false>(Kt, Vt, qf, oacc, m_i, l_i, scale_l2, lm, c, g, k0, myq, lg_row, vis_lo, vis_hi);
    else if (k0 + 32 == q0)     // first half visible, second half on the diagonal
        tile_step<D, 2, true>(Kt, Vt, qf, oacc, m_i, l_i, scale_l2, lm, c, g, k0, myq, lg_row, vis_lo, vis_hi);
    else                        // k0 == q0: first half on the diagonal, second half above it
        tile_step<D, 1, true>(Kt, Vt, qf, oacc, m_i, l_i, scale_l2, lm, c, g, k0, myq, lg_row, vis_lo, vis_hi);
}

// One-dimensional grid of ceil(n/128) * H * B workgroups (the mapping to query tile and strip is in the kernel).
// Register budget: two waves per SIMD (256 registers each; the kernel takes 214), i.e. two workgroups
// per compute unit: while one waits for a tile, a barrier or its first loads, the other one runs.
// (MFMA and VALU work of the two waves of a SIMD add up rather than overlap on this part: measured.)
template <int D>
__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(PrefillArgs a) {
    using L = TileLayout<D>;
    constexpr int KS = D / 16;          // contraction steps of S^T
    constexpr int DT = D / 32;          // 32-row tiles of O^T
    // two buffers as two objects, so that the compiler can tell a direct load into one from the reads of the other
    __shared__ __attribute__((aligned(1024))) uint16_t buf0[2 * L::TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t buf1[2 * L::TILE];

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
    // Query tiles are cut from the END of the prompt in whole 32-row blocks: the blocks that a prompt
    // of no multiple of 128 rows leaves empty then sit at the front of a strip's FIRST tile, the one
    // that walks the fewest key tiles, and not behind its last (the one that walks them all).  Such a
    // wave has q0 < 0 and only helps to load tiles.  (Blocks stay aligned to 32 rows and key tiles to
    // 64, which is what the diagonal handling relies on.)
    const int q0 = qt * kBM + wave * 32 - a.q_shift;
    const int myq = q0 + c;
    const int64_t bh = (int64_t)b * a.H + h;

    const uint16_t* Qp = reinterpret_cast<const uint16_t*>(a.q) + b * a.q_sb + h * a.q_sh;
    const uint16_t* Kp = reinterpret_cast<const uint16_t*>(a.k) + b * a.k_sb + h * a.k_sh;
    const uint16_t* Vp = reinterpret_cast<const uint16_t*>(a.v) + b * a.v_sb + h * a.v_sh;

    // this lane's part of the direct loads' source: row (wave * RPI + lane / UPR) of a 1 KB group, and the
    // 16-byte unit that the permutation assigns to its LDS slot (the permutations repeat every RPI * 4
    // rows or sooner, so they are the same for every group and every tile), as a byte offset
    uint32_t k_lane, v_lane;
    {
        const int row0 = wave * L::RPI + lane / L::UPR, u = lane % L::UPR;
        const int rowc = min(row0, n - 1);              // a prompt shorter than one group of rows
        k_lane = (uint32_t)(2 * (rowc * a.k_st + (u ^ L::k_swz(row0)) * 8));
        v_lane = (uint32_t)(2 * (rowc * a.v_st + (u ^ L::v_swz(row0)) * 8));
    }
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);     // for scalar address arithmetic only
    const uint32_t lds0 = lds_addr(buf0), lds1 = lds_addr(buf1);
    issue_tile<D>(lds0, Kp, Vp, k_lane, v_lane, a.k_st, a.v_st, 0, n, lane, wave, wave_s);
    Frag qf[KS];
    {
        const uint16_t* qrow = Qp + (int64_t)max(0, min(myq, n - 1)) * a.q_st;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s].u4 = *reinterpret_cast<const u32x4*>(qrow + 16 * s + 8 * g);
    }
    LaneMap<D> lm;
    lm.init(c, g);
    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    float m_i = -INFINITY, l_i = 0.f;

    // window rows (the last W queries) held by this wave?
    const bool wave_has_window = a.pre_logits != nullptr && q0 + 31 >= n - a.window && q0 < n && q0 >= 0;
    const int w_idx = myq - (n - a.window);
    const bool lane_in_window = wave_has_window && w_idx >= 0 && myq < n;
    float* lg_row = lane_in_window ? a.pre_logits + (bh * a.window + w_idx) * a.vis_len : nullptr;
    const int vis_lo = a.sys_len, vis_hi = a.sys_len + a.vis_len;

    const int k_end = min(n, qt * kBM + kBM - a.q_shift);   // keys this workgroup can see
    const int nt = (k_end + kBN - 1) / kBN;
    const bool wave_live = q0 >= 0 && q0 < n;           // else all 32 queries lie outside the prompt
    wait_direct_loads();
    __syncthreads();
    // Tiles alternate between the buffers; the loop body handles one pair.  A buffer is refilled one
    // iteration after its last read, and every wave has passed a barrier in between.
    for (int t = 0; t < nt; t += 2) {
        if (t + 1 < nt) issue_tile<D>(lds1, Kp, Vp, k_lane, v_lane, a.k_st, a.v_st, (t + 1) * kBN, n, lane, wave, wave_s);
        if (wave_live && t * kBN <= q0)                 // else the tile lies entirely above this wave's diagonal
            consume_tile<D>(buf0, t * kBN, q0, qf, oacc, m_i, l_i, a.scale_l2, lm, c, g, myq, lg_row, vis_lo, vis_hi);
        wait_direct_loads();
        __syncthreads();
        if (t + 1 >= nt) break;
        if (t + 2 < nt) issue_tile<D>(lds0, Kp, Vp, k_lane, v_lane, a.k_st, a.v_st, (t + 2) * kBN, n, lane, wave, wave_s);
        if (wave_live && (t + 1) * kBN <= q0)
            consume_tile<D>(buf1, (t + 1) * kBN, q0, qf, oacc, m_i, l_i, a.scale_l2, lm, c, g, myq, lg_row, vis_lo, vis_hi);
        wait_direct_loads();
        __syncthreads();
    }
    // ---- normalise and store -----------------------------------------------------------------
    float l_lo, l_hi;
    both_halves(l_i, l_lo, l_hi);
    const float l_tot = l_lo + l_hi;
    const float rl = 1.0f / l_tot;
    // The accumulator holds O transposed (a lane owns one query and, per register quad, 4 consecutive
    // columns): stored straight from there, a wave-wide store would touch 32 rows with 8 bytes each.
    // So the wave's 32 x D block goes through LDS (both tile buffers are free after the last barrier;
    // each wave uses a region of its own) and leaves as whole rows, 16 bytes per lane.
    {
        constexpr int OSTR = D + 8;                     // padded row, 16-byte aligned
        constexpr int VPR = D / 8;                      // 16-byte vectors (lanes) per row
        constexpr int RPI = 64 / VPR;                   // rows per wave-wide store
        uint16_t* obuf = (wave < 2 ? buf0 : buf1) + (wave & 1) * (32 * OSTR);
        static_assert(2 * 32 * OSTR <= 2 * L::TILE, "two waves' output blocks fit one tile buffer");
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int dd = 32 * dt + 8 * rq + 4 * g;
                const f32x2 o01 = {oacc[dt][4 * rq] * rl, oacc[dt][4 * rq + 1] * rl};
                const f32x2 o23 = {oacc[dt][4 * rq + 2] * rl, oacc[dt][4 * rq + 3] * rl};
                uint2 pk;                               // packed conversion, round to nearest even
                pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(o01, bf16x2));
                pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(o23, bf16x2));
                *reinterpret_cast<uint2*>(obuf + c * OSTR + dd) = pk;
            }
        uint16_t* obase = reinterpret_cast<uint16_t*>(a.out) + b * a.o_sb + h * a.o_sh;
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int r = i * RPI + lane / VPR;
            const u32x4 val = *reinterpret_cast<const u32x4*>(obuf + r * OSTR + (lane % VPR) * 8);
            if (wave_live && q0 + r < n) *reinterpret_cast<u32x4*>(obase + (int64_t)(q0 + r) * a.o_st + (lane % VPR) * 8) = val;
        }
    }
    if (myq < n) {
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
    pa.q_shift = (pa.n_qt * kBM - a.n) / 32 * 32;       // whole empty 32-row blocks, moved to the front
    pa.B = B;
    const int64_t wgs = (int64_t)pa.n_qt * a.H * B;
    if (wgs > 0x7fffffff) return ST3_ERR_UNSUPPORTED;
    // the direct loads address a strip as a scalar base plus a 32-bit byte offset
    if ((int64_t)a.n * a.k_st * 2 >= (int64_t)1 << 31 || (int64_t)a.n * a.v_st * 2 >= (int64_t)1 << 31) return ST3_ERR_UNSUPPORTED;
    dim3 grid((unsigned)wgs);
    if (D == 128) prefill_mfma_kernel<128><<<grid, 256, 0, st>>>(pa);
    else if (D == 64) prefill_mfma_kernel<64><<<grid, 256, 0, st>>>(pa);
    else return ST3_ERR_UNSUPPORTED;
    return ST3_OK;
}

}  // namespace st3
