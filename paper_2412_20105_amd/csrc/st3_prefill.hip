// Prefill attention (Eq. 2, causal) with the visual mass of the last query rows (Sec. 3.2).
//
// Two kernels produce the attention output:
//   * prefill_rows_kernel  - float32 arithmetic on any supported element type, one wavefront per
//                            query row streaming the keys it may see.  Used for float32 inputs.
//   * prefill_mfma_kernel  - bf16 inputs, MFMA contraction with LDS-staged K/V tiles (st3_prefill_mfma.hip).
// Both leave, for the last W query rows, the scaled logits of the visual keys and the row's
// (max, sum) in the workspace; prefill_mass_kernel turns them into probabilities and adds them
// over heads and rows in a fixed order.
#include "st3_attend.h"
#include "st3_prefill.h"

namespace st3 {

namespace {

constexpr int kRowsPerBlock = 4;

// grid (ceil(n/4), H, B); wave w of block x handles query row n-1-(4x+w): longest rows first.
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_rows_kernel(PrefillArgs a) {
    using M = RowMap<T, D>;
    constexpr int EPL = M::EPL, LPR = M::LPR;
    const int h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int i = a.n - 1 - ((int)blockIdx.x * kRowsPerBlock + wave);
    if (i < 0) return;
    const T* qrow = reinterpret_cast<const T*>(a.q) + b * a.q_sb + h * a.q_sh + (int64_t)i * a.q_st;
    const T* kbase = reinterpret_cast<const T*>(a.k) + b * a.k_sb + h * a.k_sh;
    const T* vbase = reinterpret_cast<const T*>(a.v) + b * a.v_sb + h * a.v_sh;
    float qf[EPL];
    load_q_slice<T, D>(qrow, lane, qf);
    WaveState<EPL> st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) st.acc[e] = 0.f;
    const int64_t bh = (int64_t)b * a.H + h;
    const int w_idx = i - (a.n - a.window);
    float* lg = nullptr;
    if (a.pre_logits && w_idx >= 0) lg = a.pre_logits + (bh * a.window + w_idx) * a.vis_len;
    // K and V may have different strides; wave_attend takes one stride, so require equality here
    wave_attend<T, D, 4, false>(qf, kbase, vbase, a.k_st, 0, i + 1, 4 * M::RPL, 0, a.scale_l2, lane, st, lg, a.sys_len,
                         a.sys_len + a.vis_len);
    finish_wave<T, D>(st);
    if (lane < LPR) {
        float o[EPL];
        const float rl = 1.0f / st.l;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] = st.acc[e] * rl;
        T* orow = reinterpret_cast<T*>(a.out) + b * a.o_sb + h * a.o_sh + (int64_t)i * a.o_st;
        *reinterpret_cast<uint4*>(orow + lane * EPL) = ElemTraits<T>::pack(o);
    }
    if (lg && lane == 0) {
        a.pre_ml[(bh * a.window + w_idx) * 2] = st.m;
        a.pre_ml[(bh * a.window + w_idx) * 2 + 1] = st.l;
    }
}

struct PrefillMassArgs {
    const float* pre_logits;
    const float* pre_ml;
    float* mass;
    int64_t mass_stride;
    int32_t n, sys_len, vis_len, window, H;
};

// grid (ceil(vis_len/128), B).  mass[b,j] = (1/H) sum_h sum_w p_{h,w}[sys_len+j]; a window row
// that precedes key sys_len+j cannot see it (causal mask) and contributes nothing.
__global__ __launch_bounds__(128) void prefill_mass_kernel(PrefillMassArgs a) {
    const int b = blockIdx.y;
    const int j = blockIdx.x * 128 + threadIdx.x;
    if (j >= a.vis_len) return;
    float acc = 0.f;
    for (int h = 0; h < a.H; ++h) {
        const int64_t bh = (int64_t)b * a.H + h;
        for (int w = 0; w < a.window; ++w) {
            const int i = a.n - a.window + w;
            if (a.sys_len + j > i) continue;
            const int64_t row = bh * a.window + w;
            float s = a.pre_logits[row * a.vis_len + j];
            acc += exp2_fast(s - a.pre_ml[row * 2]) / a.pre_ml[row * 2 + 1];
        }
    }
    a.mass[(int64_t)b * a.mass_stride + j] = acc / (float)a.H;
}

template <typename T, int D>
void launch_rows(const PrefillArgs& a, int B, hipStream_t st) {
    dim3 grid((a.n + kRowsPerBlock - 1) / kRowsPerBlock, a.H, B);
    prefill_rows_kernel<T, D><<<grid, 256, 0, st>>>(a);
}

bool tensor_ok(const st3_tensor4* t, int eb, int d) {
    if (!t || !t->data || !aligned16(t->data)) return false;
    if (t->stride_t < d || t->stride_h < 0 || t->stride_b < 0) return false;
    return (t->stride_t * eb) % 16 == 0 && (t->stride_h * eb) % 16 == 0 && (t->stride_b * eb) % 16 == 0;
}

}  // namespace
}  // namespace st3

extern "C" st3_status st3_prefill_attention(const st3_attn_shape* shape, const st3_tensor4* q, const st3_tensor4* k,
                                            const st3_tensor4* v, int32_t n, int32_t sys_len, int32_t vis_len,
                                            int32_t score_window, const st3_tensor4* out, float* vis_mass,
                                            int64_t mass_stride, void* workspace, size_t workspace_bytes,
                                            void* stream) {
    using namespace st3;
    st3_status s = check_shape(shape);
    if (s != ST3_OK) return s;
    const int B = shape->batch, H = shape->heads, D = shape->head_dim, eb = elem_bytes(shape->dtype);
    if (!tensor_ok(q, eb, D) || !tensor_ok(k, eb, D) || !tensor_ok(v, eb, D) || !tensor_ok(out, eb, D))
        return ST3_ERR_INVALID_ARG;
    if (n <= 0 || sys_len < 0 || vis_len < 0 || sys_len + vis_len > n) return ST3_ERR_INVALID_ARG;
    if (n > 32768) return ST3_ERR_UNSUPPORTED;
    if (score_window < 1 || score_window > n || score_window > kMaxWindow) return ST3_ERR_INVALID_ARG;
    if (k->stride_t != v->stride_t) return ST3_ERR_UNSUPPORTED;
    const bool want_mass = vis_mass != nullptr && vis_len > 0;
    if (want_mass && mass_stride < vis_len) return ST3_ERR_INVALID_ARG;
    const PrefillWs wl = prefill_ws(B, H, vis_len, score_window);
    // the prefill scratch sits at the END of the workspace, clear of the decode-path region
    if (want_mass) {
        if (!workspace || !aligned16(workspace)) return ST3_ERR_INVALID_ARG;
        if (workspace_bytes < wl.total) return ST3_ERR_WORKSPACE_TOO_SMALL;
    }
    const size_t ws_base = want_mass ? (workspace_bytes - wl.total) / 256 * 256 : 0;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    PrefillArgs a{};
    a.q = q->data; a.k = k->data; a.v = v->data; a.out = out->data;
    a.q_sb = q->stride_b; a.q_sh = q->stride_h; a.q_st = q->stride_t;
    a.k_sb = k->stride_b; a.k_sh = k->stride_h; a.k_st = k->stride_t;
    a.v_sb = v->stride_b; a.v_sh = v->stride_h; a.v_st = v->stride_t;
    a.o_sb = out->stride_b; a.o_sh = out->stride_h; a.o_st = out->stride_t;
    a.n = n; a.sys_len = sys_len; a.vis_len = vis_len; a.window = score_window; a.H = H;
    a.scale_l2 = scale_log2(shape);
    if (want_mass) {
        char* ws = reinterpret_cast<char*>(workspace) + ws_base;
        a.pre_logits = reinterpret_cast<float*>(ws + wl.pre_logits);
        a.pre_ml = reinterpret_cast<float*>(ws + wl.pre_ml);
    }
    // diagnostic override of the kernel choice (0 unless the debug block is enabled): 1 = the row
    // kernel also for bf16, 2 = the MFMA kernel or fail
    const int g_prefill_path = debug_state().prefill_path;
    bool use_mfma = shape->dtype == ST3_BF16;
    if (g_prefill_path == 1) use_mfma = false;
    if (g_prefill_path == 2 && shape->dtype != ST3_BF16) return ST3_ERR_UNSUPPORTED;
    if (use_mfma) {
        s = launch_prefill_mfma(a, B, D, st);
        if (s == ST3_ERR_UNSUPPORTED && g_prefill_path != 2) use_mfma = false;    // shape outside the MFMA kernel
        else if (s != ST3_OK) return s;
    }
    if (!use_mfma) {
        if (shape->dtype == ST3_BF16) {
            if (D == 128) launch_rows<bf16_t, 128>(a, B, st); else launch_rows<bf16_t, 64>(a, B, st);
        } else {
            if (D == 128) launch_rows<float, 128>(a, B, st); else launch_rows<float, 64>(a, B, st);
        }
    }
    if (want_mass) {
        PrefillMassArgs m{a.pre_logits, a.pre_ml, vis_mass, mass_stride, n, sys_len, vis_len, score_window, H};
        prefill_mass_kernel<<<dim3((vis_len + 127) / 128, B), 128, 0, st>>>(m);
    }
    return check_launch();
}
