// Internal helpers shared by the HIP translation units of libst3 (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "st3.h"

namespace st3 {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

void set_last_hip_error(hipError_t e);

// Process-wide diagnostic switches (st3_debug_* / st3_profile_* of st3.h).  They exist in every build
// but stay at their defaults - and the calls that set them return ST3_ERR_UNSUPPORTED - unless the
// environment held ST3_DEBUG=1 when the library was loaded.  Plain ints read by the launch code;
// set them only while no other thread is inside a library call.
struct DebugState {
    bool enabled;           // ST3_DEBUG=1 at load
    int prefill_path;       // 0 = automatic, 1 = float32 row kernel, 2 = MFMA kernel or fail
    int attend_tile;        // 0 = automatic, else the forced tile size of the decode attention kernel
};
DebugState& debug_state();  // st3_api.hip
constexpr int kMaxDevices = 64;     // per-device caches (occupancy, scratch addresses) are indexed by the HIP device id

// Launch-error capture used by every entry point after enqueueing its kernels.
inline st3_status check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_hip_error(e);
        return ST3_ERR_HIP;
    }
    return ST3_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int elem_bytes(int dtype) { return dtype == ST3_BF16 ? 2 : dtype == ST3_E4M3 ? 1 : 4; }
// bytes of one cache element of a layer
inline int kv_elem_bytes(const st3_attn_shape* s, const st3_kv_layer* kv) {
    return kv->format == ST3_KV_E4M3 ? 1 : elem_bytes(s->dtype);
}

// Validates what every attention entry point needs from `shape`.
inline st3_status check_shape(const st3_attn_shape* s) {
    if (!s) return ST3_ERR_INVALID_ARG;
    if (s->batch <= 0 || s->heads <= 0) return ST3_ERR_INVALID_ARG;
    if (s->dtype != ST3_F32 && s->dtype != ST3_BF16) return ST3_ERR_UNSUPPORTED;
    if (s->head_dim != 64 && s->head_dim != 128) return ST3_ERR_UNSUPPORTED;
    if (s->heads > 1024 || s->batch > 65535) return ST3_ERR_UNSUPPORTED;
    if (!(s->softmax_scale >= 0.0f)) return ST3_ERR_INVALID_ARG;
    return ST3_OK;
}

inline float scale_log2(const st3_attn_shape* s) {
    float sc = s->softmax_scale > 0.0f ? s->softmax_scale : 1.0f / sqrtf((float)s->head_dim);
    return sc * kLog2e;
}

// ---------------------------------------------------------------------------------------------
// Workspace carving.  The decode-path region is laid out from the cache CAPACITY alone, so that
// every call on a layer's workspace sees the same offsets whatever the step's lengths are: the
// eviction plan finishes the mass from what the attend launch left there, and a lazy layer reads
// its source layer's logits and normalisers from the source's workspace.  The prefill region
// starts behind it and depends on the call's own sizes.
// ---------------------------------------------------------------------------------------------
constexpr int kMaxWindow = 16;
#ifndef ST3_DECODE_TARGET_WGS
#define ST3_DECODE_TARGET_WGS 256      // one workgroup per compute unit; 512-1024 measured 5-14 % slower at B*H = 320-512
#endif
constexpr int kDecodeTargetWgs = ST3_DECODE_TARGET_WGS;     // split the KV range until about this many workgroups exist
#ifndef ST3_DECODE_TARGET_WGS_MERGED
#define ST3_DECODE_TARGET_WGS_MERGED 1024
#endif
// ... and this many when the chunk partials are merged inside the step's plan launch, where a split costs no launch of
// its own (13B shape, attend launch: B = 4 14.1 -> 11.7 us, B = 8 21.7 -> 20.2 us; 256, 512, 1024, 1536, 2048 measured),
// unless B*H alone reaches half of it (B*H >= 512 ran the same or slower when cut)
constexpr int kDecodeTargetWgsMerged = ST3_DECODE_TARGET_WGS_MERGED;
constexpr int kDecodeTargetWgsMax = kDecodeTargetWgs > kDecodeTargetWgsMerged ? kDecodeTargetWgs : kDecodeTargetWgsMerged;
constexpr int kDecodeMaxSplit = 64;
// Largest chunk of a strip (rows): a decode_attend_kernel workgroup collects the logits it keeps in LDS, 4 bytes per row
// of its chunk at most: 16 KB, so that the seven workgroups a compute unit can hold still fit its 160 KB.
constexpr int kLogitStageMaxRows = 4096;
#ifndef ST3_DECODE_MIN_CHUNK
#define ST3_DECODE_MIN_CHUNK 64
#endif
// never cut a (b,h) strip into chunks shorter than this (32 and 96 rows measured 2-8 % slower per step at B*H = 32 and 40)
constexpr int kDecodeMinChunk = ST3_DECODE_MIN_CHUNK;

// Number of chunks each (b,h) strip is cut into for a given upper bound on its length.
inline int decode_nsplit(int B, int H, int max_kv, int target_wgs = kDecodeTargetWgs) {
    const int64_t bh = (int64_t)B * H;
    int64_t want = (target_wgs + bh - 1) / bh;
    if (target_wgs > kDecodeTargetWgs && 2 * bh >= target_wgs) want = 1;
    int64_t by_len = ((int64_t)max_kv + kDecodeMinChunk - 1) / kDecodeMinChunk;
    int64_t ns = want < by_len ? want : by_len;
    // A small even number of chunks runs slower than the odd number below it (attend launch, whole-step call, 1 / 2 / 3 /
    // 4 / 5 / 6 / 8 chunks: high-resolution prompt at batch 8, B*H = 256, 31.8 / 33.9 / 31.4 / 35.7 / 32.6 / 34.2 / 38.5 us;
    // 13B shape at batch 8, B*H = 320, 21.5 / 21.2 / 19.3 / 19.9 / 19.8 / 20.1 / 23.0 us): workgroup ids go round-robin to
    // the 8 XCDs, so with an even count a chunk index always meets the same XCDs (rotating the chunk index over the strips
    // recovers part of it, 35.7 -> 34.3 and 19.9 -> 19.3 us).  Where a cut costs a launch of its own (the lower target) one
    // chunk fewer is taken always - two chunks become none, and the merge launch goes; where it is free, only if enough
    // workgroups remain (at B*H = 40 the late, short layers of the 13B shape lost 2 % with 3 chunks instead of 4).
    if (ns > 1 && ns % 2 == 0 && (target_wgs <= kDecodeTargetWgs || bh * (ns - 1) >= 2 * kDecodeTargetWgs)) ns -= 1;
    const int64_t by_stage = ((int64_t)max_kv + kLogitStageMaxRows - 1) / kLogitStageMaxRows;      // chunks no longer than the staging area
    if (ns < by_stage) ns = by_stage;
    if (ns > kDecodeMaxSplit) ns = kDecodeMaxSplit;
    return ns < 1 ? 1 : (int)ns;
}
// Chunk length for that split count: a multiple of 32 rows.
inline int decode_chunk(int max_kv, int nsplit) {
    int c = (max_kv + nsplit - 1) / nsplit;
    c = (c + 31) / 32 * 32;
    return c < 32 ? 32 : c;
}

// A layer's attention launch can leave up to 256 bytes of the host's choosing in the layer's workspace (one workgroup stores
// them): the whole-step call passes each layer's eviction-plan arguments this way, so that ONE plan launch can serve every
// layer of the step - by value, 16 layers' arguments fill the kernel-argument block.
constexpr int kPlanStashWords = 64;
struct PlanStash {
    uint32_t w[kPlanStashWords];
    uint32_t* dst;              // DEVICE, in the layer's workspace; null: nothing to leave
};

struct DecodeWs {
    size_t part_o, part_ml, logits, pending, plan_args, moves_cnt, moves, total;
    int nsplit_cap;
    int max_moves;
};

inline DecodeWs decode_ws(int B, int H, int D, int capacity) {
    DecodeWs w{};
    if (capacity < 1) capacity = 1;
    w.nsplit_cap = decode_nsplit(B, H, capacity, kDecodeTargetWgsMax);
    w.max_moves = capacity;                 // a stable shift moves every row at most once
    size_t off = 0;
    const size_t BH = (size_t)B * H;
    w.part_o = off;     off = align_up(off + BH * w.nsplit_cap * D * sizeof(float), 256);
    w.part_ml = off;    off = align_up(off + BH * w.nsplit_cap * 2 * sizeof(float), 256);
    w.logits = off;     off = align_up(off + BH * (size_t)capacity * sizeof(float), 256);   // [B,H,capacity]
    w.pending = off;    off = align_up(off + (size_t)B * 4 * sizeof(int32_t), 256);         // [B][4]
    w.plan_args = off;  off = align_up(off + kPlanStashWords * sizeof(uint32_t), 256);       // what a PlanStash leaves
    w.moves_cnt = off;  off = align_up(off + (size_t)B * sizeof(int32_t), 256);
    w.moves = off;      off = align_up(off + (size_t)B * w.max_moves * 2 * sizeof(int32_t), 256);
    w.total = off;
    return w;
}

struct PrefillWs {
    size_t pre_logits, pre_ml, total;
};

inline PrefillWs prefill_ws(int B, int H, int vis_len, int window) {
    PrefillWs w{};
    if (vis_len < 0) vis_len = 0;
    if (window < 1) window = 1;
    const size_t BH = (size_t)B * H;
    size_t off = 0;
    w.pre_logits = off; off = align_up(off + BH * (size_t)window * vis_len * sizeof(float), 256);
    w.pre_ml = off;     off = align_up(off + BH * (size_t)window * 2 * sizeof(float), 256);
    w.total = off;
    return w;
}

// ---------------------------------------------------------------------------------------------
// Device helpers
// ---------------------------------------------------------------------------------------------
#if defined(__HIPCC__)

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// float32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> {
    static constexpr int kBytes = 4;
    static constexpr int kPerVec = 4;       // elements in a 16-byte vector
    __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
    __device__ static __forceinline__ uint4 pack(const float* f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};
struct bf16_t { uint16_t bits; };
template <> struct ElemTraits<bf16_t> {
    static constexpr int kBytes = 2;
    static constexpr int kPerVec = 8;
    __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
        f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
        f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
    }
    __device__ static __forceinline__ uint4 pack(const float* f) {
        return make_uint4(f32_to_bf16_bits(f[0]) | (f32_to_bf16_bits(f[1]) << 16),
                          f32_to_bf16_bits(f[2]) | (f32_to_bf16_bits(f[3]) << 16),
                          f32_to_bf16_bits(f[4]) | (f32_to_bf16_bits(f[5]) << 16),
                          f32_to_bf16_bits(f[6]) | (f32_to_bf16_bits(f[7]) << 16));
    }
};

// One byte per element: OCP FP8 E4M3 code.  The hardware conversion used by unpack() was checked
// against the format's definition for all 256 codes (bias 7, subnormals, S.1111.111 = NaN, 448
// largest) and takes the bytes of a word from low to high.
struct e4m3_t { uint8_t bits; };
typedef float f32x2_t __attribute__((ext_vector_type(2)));
template <> struct ElemTraits<e4m3_t> {
    static constexpr int kBytes = 1;
    static constexpr int kPerVec = 16;
    __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
            const f32x2_t hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
            f[4 * i] = lo.x; f[4 * i + 1] = lo.y; f[4 * i + 2] = hi.x; f[4 * i + 3] = hi.y;
        }
    }
};

// float32 -> E4M3 code: saturate at +-448, round to nearest, ties to the even code, sign kept
// (also of zero), NaN -> 0x7F.  Written out in integer arithmetic so that the result does not
// depend on a conversion instruction's mode bits.
__device__ __forceinline__ uint32_t f32_to_e4m3(float t) {
    const uint32_t u = __float_as_uint(t);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return 0x7fu;                      // NaN
    if (a >= 0x43e00000u) return sign | 0x7eu;              // |t| >= 448 (infinity included)
    if (a < 0x3c800000u) {                                  // |t| < 2^-6: multiples of 2^-9, code = the multiple
        const float m = rintf(__uint_as_float(a) * 512.0f); // exact product, round half to even; 8 carries into 2^-6
        return sign | (uint32_t)m;
    }
    const uint32_t e = (a >> 23) - 127u + 7u;               // 1 .. 15
    const uint32_t mant = a & 0x7fffffu;
    uint32_t code = (e << 3) | (mant >> 20);
    const uint32_t rem = mant & 0xfffffu;
    code += (rem > 0x80000u || (rem == 0x80000u && (code & 1u))) ? 1u : 0u;     // carry runs into the exponent
    return sign | code;
}

// x / scale as the quantiser defines it: one correctly rounded float32 division.
__device__ __forceinline__ uint32_t quantize_e4m3(float x, float scale) { return f32_to_e4m3(__fdiv_rn(x, scale)); }

// x of this lane and x of lane ^ OFF, as the pair (a, b) in an order that depends on the lane: enough
// for any symmetric combination (max, sum).  OFF = 32 and 16 use the swap instructions of gfx950
// (v_permlane32_swap trades lanes 32..63 of its first operand for lanes 0..31 of its second,
// v_permlane16_swap does the same with the odd and even rows of 16 lanes; with both operands x one
// result holds the lower partner's value in both places and the other the upper partner's): no LDS
// round trip, which a shuffle across rows of 16 lanes takes.
template <int OFF>
__device__ __forceinline__ void lane_pair(float x, float& a, float& b) {
    if constexpr (OFF == 32) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
        a = __uint_as_float(r[0]); b = __uint_as_float(r[1]);
    } else if constexpr (OFF == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
        a = __uint_as_float(r[0]); b = __uint_as_float(r[1]);
    } else {
        a = x; b = __shfl_xor(x, OFF);
    }
}
template <int OFF>
__device__ __forceinline__ float pair_max(float x) { float a, b; lane_pair<OFF>(x, a, b); return fmaxf(a, b); }
template <int OFF>
__device__ __forceinline__ float pair_sum(float x) { float a, b; lane_pair<OFF>(x, a, b); return a + b; }

// Sum over aligned groups of G consecutive lanes (G in {4,8,16,32}); every lane of a group ends
// with the group's total.  Steps below 16 lanes use DPP row operations; they rely on all lanes
// of the already-reduced sub-group holding the same value, so a mirror acts as the XOR step.
template <int G>
__device__ __forceinline__ float group_sum(float v) {
    // xor 1, xor 2 inside a quad
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    if (G >= 8)   // row_half_mirror: lane i <-> 7-i within 8 lanes
        v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    if (G >= 16)  // row_mirror: lane i <-> 15-i within 16 lanes
        v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
    if (G >= 32) v = pair_sum<16>(v);
    return v;
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// Maximum / sum over the lanes l, l ^ FROM, l ^ 2 FROM, ... up to the whole wave of 64.
template <int FROM>
__device__ __forceinline__ float wave_max_from(float x) {
    if constexpr (FROM <= 1) x = pair_max<1>(x);
    if constexpr (FROM <= 2) x = pair_max<2>(x);
    if constexpr (FROM <= 4) x = pair_max<4>(x);
    if constexpr (FROM <= 8) x = pair_max<8>(x);
    if constexpr (FROM <= 16) x = pair_max<16>(x);
    return pair_max<32>(x);
}
template <int FROM>
__device__ __forceinline__ float wave_sum_from(float x) {
    if constexpr (FROM <= 1) x = pair_sum<1>(x);
    if constexpr (FROM <= 2) x = pair_sum<2>(x);
    if constexpr (FROM <= 4) x = pair_sum<4>(x);
    if constexpr (FROM <= 8) x = pair_sum<8>(x);
    if constexpr (FROM <= 16) x = pair_sum<16>(x);
    return pair_sum<32>(x);
}

#endif  // __HIPCC__

}  // namespace st3
