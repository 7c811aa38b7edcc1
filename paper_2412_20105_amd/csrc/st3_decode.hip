// Decode attention over a ragged KV cache with fused visual-mass output, KV append, and the
// merge kernel that finishes both (Eq. 2 with a single query row; score extraction of Sec. 3.2).
#include "st3_attend.h"

namespace st3 {

void profile_mark(hipStream_t st, bool after);     // st3_api.hip

namespace {

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = kDecodeThreads / kWave;
constexpr int kKeysPerWave = kDecodeChunk / kDecodeWaves;

struct DecodeArgs {
    const void* q;
    const void* k;
    const void* v;
    int64_t stride_b, stride_h, stride_t;
    const int32_t* kv_len;
    const int32_t* vis_len;
    int32_t sys_len, max_vis, max_kv, H, nsplit_max;
    float scale_l2;
    float* part_o;
    float* part_ml;
    float* logits;          // null when no mass is wanted
};

// grid (nsplit_max, H, B); one workgroup = one chunk of kDecodeChunk keys of one (b,h).
template <typename T, int D, int U>
__global__ __launch_bounds__(kDecodeThreads) void decode_split_kernel(DecodeArgs a) {
    using M = RowMap<T, D>;
    constexpr int EPL = M::EPL, LPR = M::LPR;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int len = min(a.kv_len[b], a.max_kv);      // never trust a device length past the host bound
    const int c0 = split * kDecodeChunk;
    if (c0 >= len) return;
    const int c1 = min(c0 + kDecodeChunk, len);
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;

    const int64_t bh = (int64_t)b * a.H + h;
    const T* qrow = reinterpret_cast<const T*>(a.q) + bh * D;
    const T* kbase = reinterpret_cast<const T*>(a.k) + b * a.stride_b + h * a.stride_h;
    const T* vbase = reinterpret_cast<const T*>(a.v) + b * a.stride_b + h * a.stride_h;

    float qf[EPL];
    load_q_slice<T, D>(qrow, lane, qf);

    WaveState<EPL> st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) st.acc[e] = 0.f;

    const int r0 = c0 + wave * kKeysPerWave;
    const int r1 = min(r0 + kKeysPerWave, c1);
    if (r0 < r1) {
        float* lg = a.logits ? a.logits + bh * a.max_vis : nullptr;
        int vis_lo = a.sys_len, vis_hi = a.sys_len + min(a.vis_len[b], a.max_vis);
        wave_attend<T, D, U>(qf, kbase, vbase, a.stride_t, r0, r1, a.scale_l2, lane, st, lg, vis_lo, vis_hi);
        finish_wave<T, D>(st);
    }

    __shared__ float sm_acc[kDecodeWaves][D];
    __shared__ float sm_m[kDecodeWaves], sm_l[kDecodeWaves];
    if (lane < LPR) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sm_acc[wave][lane * EPL + e] = st.acc[e];
    }
    if (lane == 0) { sm_m[wave] = st.m; sm_l[wave] = st.l; }
    __syncthreads();
    if (tid < D) {
        float m = sm_m[0];                              // wave 0 always has rows: finite
#pragma unroll
        for (int w = 1; w < kDecodeWaves; ++w) m = fmaxf(m, sm_m[w]);
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            float f = exp2_fast(sm_m[w] - m);           // empty wave: exp2(-inf) = 0
            o = fmaf(sm_acc[w][tid], f, o);
            l = fmaf(sm_l[w], f, l);
        }
        const int64_t slot = bh * a.nsplit_max + split;
        a.part_o[slot * D + tid] = o;
        if (tid == 0) { a.part_ml[slot * 2] = m; a.part_ml[slot * 2 + 1] = l; }
    }
}

struct MergeArgs {
    const float* part_o;
    const float* part_ml;
    const float* logits;
    const int32_t* kv_len;
    const int32_t* vis_len;
    int32_t H, nsplit_max, max_vis, max_kv;
    void* out;
    float* mass;            // null: no mass
    int64_t mass_stride;
};

constexpr int kMergeThreads = 128;

// grid (H + mass_blocks, B).  Blocks y < H merge the split partials of head y into out[b,y,:].
// Blocks y >= H produce 128 mass entries each: they first rebuild (m_h, l_h) for every head,
// then add the heads in index order, so the sum is the same on every run.
template <typename T, int D>
__global__ __launch_bounds__(kMergeThreads) void decode_merge_kernel(MergeArgs a) {
    const int b = blockIdx.y, tid = threadIdx.x;
    const int len = min(a.kv_len[b], a.max_kv);
    const int ns = (len + kDecodeChunk - 1) / kDecodeChunk;
    if ((int)blockIdx.x < a.H) {
        const int h = blockIdx.x;
        const int64_t bh = (int64_t)b * a.H + h;
        if (tid >= D) return;
        float o = 0.f;
        if (ns > 0) {
            const float* ml = a.part_ml + bh * a.nsplit_max * 2;
            float m = ml[0];
            for (int s = 1; s < ns; ++s) m = fmaxf(m, ml[2 * s]);
            float l = 0.f;
            for (int s = 0; s < ns; ++s) {
                float f = exp2_fast(ml[2 * s] - m);
                l = fmaf(ml[2 * s + 1], f, l);
                o = fmaf(a.part_o[(bh * a.nsplit_max + s) * D + tid], f, o);
            }
            o = o / l;
        }
        if (sizeof(T) == 4) reinterpret_cast<float*>(a.out)[bh * D + tid] = o;
        else reinterpret_cast<uint16_t*>(a.out)[bh * D + tid] = (uint16_t)f32_to_bf16_bits(o);
        return;
    }
    if (a.mass == nullptr) return;
    __shared__ float sm_m[1024], sm_rl[1024];
    for (int h = tid; h < a.H; h += kMergeThreads) {
        const float* ml = a.part_ml + ((int64_t)b * a.H + h) * a.nsplit_max * 2;
        float m = -INFINITY, l = 0.f;
        if (ns > 0) {
            m = ml[0];
            for (int s = 1; s < ns; ++s) m = fmaxf(m, ml[2 * s]);
            for (int s = 0; s < ns; ++s) l = fmaf(ml[2 * s + 1], exp2_fast(ml[2 * s] - m), l);
        }
        sm_m[h] = m;
        sm_rl[h] = ns > 0 ? 1.0f / l : 0.f;
    }
    __syncthreads();
    const int j = (blockIdx.x - a.H) * kMergeThreads + tid;
    const int nv = min(a.vis_len[b], a.max_vis);
    if (j >= nv) return;
    float acc = 0.f;
    for (int h = 0; h < a.H; ++h) {
        float s = a.logits[((int64_t)b * a.H + h) * a.max_vis + j];
        acc += exp2_fast(s - sm_m[h]) * sm_rl[h];
    }
    a.mass[(int64_t)b * a.mass_stride + j] = acc / (float)a.H;
}

struct AppendArgs {
    void* k;
    void* v;
    int64_t stride_b, stride_h, stride_t;
    const void* k_new;
    const void* v_new;
    const int32_t* kv_len;
    int32_t H, capacity;
};

// grid (H, B), 64 threads: lanes [0, LPR) copy the K row, lanes [LPR, 2*LPR) the V row.
template <typename T, int D>
__global__ __launch_bounds__(64) void append_kernel(AppendArgs a) {
    using M = RowMap<T, D>;
    const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const int row = a.kv_len[b];
    if (row >= a.capacity || lane >= 2 * M::LPR) return;
    const bool is_v = lane >= M::LPR;
    const int c = (lane % M::LPR) * M::EPL;
    const int64_t bh = (int64_t)b * a.H + h;
    const T* src = reinterpret_cast<const T*>(is_v ? a.v_new : a.k_new) + bh * D + c;
    T* dst = reinterpret_cast<T*>(is_v ? a.v : a.k) + b * a.stride_b + h * a.stride_h + row * a.stride_t + c;
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
}

__global__ void bump_len_kernel(int32_t* kv_len, int32_t B, int32_t capacity) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B && kv_len[b] < capacity) kv_len[b] += 1;
}

template <typename T, int D>
void launch_decode(const DecodeArgs& da, const MergeArgs& ma, int B, hipStream_t st) {
    dim3 g1(da.nsplit_max, da.H, B);
    profile_mark(st, false);
    decode_split_kernel<T, D, 8><<<g1, kDecodeThreads, 0, st>>>(da);
    profile_mark(st, true);
    int mass_blocks = ma.mass ? (ma.max_vis + kMergeThreads - 1) / kMergeThreads : 0;
    dim3 g2(ma.H + mass_blocks, B);
    decode_merge_kernel<T, D><<<g2, kMergeThreads, 0, st>>>(ma);
}

template <typename T, int D>
void launch_append(const AppendArgs& aa, int B, int32_t* kv_len, hipStream_t st) {
    append_kernel<T, D><<<dim3(aa.H, B), 64, 0, st>>>(aa);
    bump_len_kernel<<<(B + 255) / 256, 256, 0, st>>>(kv_len, B, aa.capacity);
}

st3_status check_kv(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg) {
    if (!kv || !seg || !kv->k || !kv->v || !seg->kv_len || !seg->vis_len) return ST3_ERR_INVALID_ARG;
    if (kv->capacity <= 0 || seg->sys_len < 0 || seg->max_vis_len < 0 || seg->max_kv_len < 0)
        return ST3_ERR_INVALID_ARG;
    if (seg->max_kv_len > kv->capacity) return ST3_ERR_INVALID_ARG;
    if (seg->sys_len + seg->max_vis_len > kv->capacity) return ST3_ERR_INVALID_ARG;
    if (kv->stride_t < s->head_dim || kv->stride_h < 0 || kv->stride_b < 0) return ST3_ERR_INVALID_ARG;
    const int eb = elem_bytes(s->dtype);
    if (!aligned16(kv->k) || !aligned16(kv->v)) return ST3_ERR_INVALID_ARG;
    if ((kv->stride_t * eb) % 16 || (kv->stride_h * eb) % 16 || (kv->stride_b * eb) % 16)
        return ST3_ERR_INVALID_ARG;
    return ST3_OK;
}

}  // namespace

// Used by st3_decode_layer_step as well.
st3_status enqueue_decode(const st3_attn_shape* shape, const void* q, const st3_kv_layer* kv,
                          const st3_segments* seg, int32_t max_kv_len, void* out, float* vis_mass,
                          int64_t mass_stride, void* workspace, size_t workspace_bytes, hipStream_t st) {
    const int B = shape->batch, H = shape->heads, D = shape->head_dim;
    WorkspaceLayout wl = workspace_layout(B, H, D, max_kv_len, seg->max_vis_len, 0, 1);
    if (workspace_bytes < wl.total) return ST3_ERR_WORKSPACE_TOO_SMALL;
    char* ws = reinterpret_cast<char*>(workspace);
    DecodeArgs da{};
    da.q = q; da.k = kv->k; da.v = kv->v;
    da.stride_b = kv->stride_b; da.stride_h = kv->stride_h; da.stride_t = kv->stride_t;
    da.kv_len = seg->kv_len; da.vis_len = seg->vis_len;
    da.sys_len = seg->sys_len; da.max_vis = seg->max_vis_len; da.max_kv = max_kv_len; da.H = H; da.nsplit_max = wl.nsplit_max;
    da.scale_l2 = scale_log2(shape);
    da.part_o = reinterpret_cast<float*>(ws + wl.part_o);
    da.part_ml = reinterpret_cast<float*>(ws + wl.part_ml);
    da.logits = (vis_mass && seg->max_vis_len > 0) ? reinterpret_cast<float*>(ws + wl.logits) : nullptr;
    MergeArgs ma{};
    ma.part_o = da.part_o; ma.part_ml = da.part_ml; ma.logits = da.logits;
    ma.kv_len = seg->kv_len; ma.vis_len = seg->vis_len;
    ma.H = H; ma.nsplit_max = wl.nsplit_max; ma.max_vis = seg->max_vis_len; ma.max_kv = max_kv_len;
    ma.out = out; ma.mass = da.logits ? vis_mass : nullptr; ma.mass_stride = mass_stride;
    if (shape->dtype == ST3_BF16) {
        if (D == 128) launch_decode<bf16_t, 128>(da, ma, B, st); else launch_decode<bf16_t, 64>(da, ma, B, st);
    } else {
        if (D == 128) launch_decode<float, 128>(da, ma, B, st); else launch_decode<float, 64>(da, ma, B, st);
    }
    return check_launch();
}

st3_status enqueue_append(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                          const void* k_new, const void* v_new, hipStream_t st) {
    const int B = shape->batch, H = shape->heads, D = shape->head_dim;
    AppendArgs aa{};
    aa.k = kv->k; aa.v = kv->v;
    aa.stride_b = kv->stride_b; aa.stride_h = kv->stride_h; aa.stride_t = kv->stride_t;
    aa.k_new = k_new; aa.v_new = v_new; aa.kv_len = seg->kv_len; aa.H = H; aa.capacity = kv->capacity;
    if (shape->dtype == ST3_BF16) {
        if (D == 128) launch_append<bf16_t, 128>(aa, B, seg->kv_len, st); else launch_append<bf16_t, 64>(aa, B, seg->kv_len, st);
    } else {
        if (D == 128) launch_append<float, 128>(aa, B, seg->kv_len, st); else launch_append<float, 64>(aa, B, seg->kv_len, st);
    }
    return check_launch();
}

st3_status validate_kv(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg) {
    return check_kv(s, kv, seg);
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
    return st3::enqueue_decode(shape, q, kv, seg, seg->max_kv_len, out, vis_mass, mass_stride, workspace,
                               workspace_bytes, reinterpret_cast<hipStream_t>(stream));
}

extern "C" st3_status st3_kv_append(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                                    const void* k_new, const void* v_new, void* stream) {
    st3_status s = st3::check_shape(shape);
    if (s != ST3_OK) return s;
    s = st3::validate_kv(shape, kv, seg);
    if (s != ST3_OK) return s;
    if (!k_new || !v_new || !st3::aligned16(k_new) || !st3::aligned16(v_new)) return ST3_ERR_INVALID_ARG;
    if (seg->max_kv_len >= kv->capacity) return ST3_ERR_INVALID_ARG;
    return st3::enqueue_append(shape, kv, seg, k_new, v_new, reinterpret_cast<hipStream_t>(stream));
}
