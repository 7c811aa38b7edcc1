// st3_decode_attention_noalloc: the decode attention for callers that cannot allocate device
// memory or carry a workspace (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc).  Same kernels as st3_decode_attention; what that call keeps in the caller's
// workspace (chunk partials, the logits of the visual keys, the per-sequence descriptors) lives
// here in one file-scope device array per GPU.
#include <mutex>

#include "st3_common.h"

namespace st3 {

st3_status validate_kv(const st3_attn_shape* s, const st3_kv_layer* kv, const st3_segments* seg);
st3_status enqueue_decode(const st3_attn_shape* shape, const void* q, const st3_kv_layer* kv,
                          const st3_segments* seg, int32_t max_kv_len, const void* k_new, const void* v_new,
                          void* out, float* vis_mass, int64_t mass_stride, bool want_mass, bool defer_mass,
                          bool keep_all_logits, void* workspace, size_t workspace_bytes, hipStream_t st,
                          bool defer_merge = false, const PlanStash* stash = nullptr);
bool decode_is_split(const st3_attn_shape* shape, const st3_kv_layer* kv, int32_t max_kv_len);

namespace {

// Every GPU the library runs on holds its own copy of this array from the moment the code object is
// loaded until the process ends.  In host code the name is only a handle for hipGetSymbolAddress:
// kernels and copies get the device address that call returns, never the name itself.
constexpr size_t kScratchBytes = ST3_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each device, once looked up

// Address of the current device's copy of `scratch` (looked up once per device, with that device
// current, which it is: the caller's buffers and stream live on it).
st3_status scratch_for_current_device(void** ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_last_hip_error(e); return ST3_ERR_HIP; }
    if (dev < 0 || dev >= kMaxDevices) return ST3_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) {
            set_last_hip_error(e);
            return ST3_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return ST3_OK;
}

}  // namespace
}  // namespace st3

extern "C" st3_status st3_decode_attention_noalloc(const st3_attn_shape* shape, const void* q, const st3_kv_layer* kv,
                                                   const st3_segments* seg, void* out, float* vis_mass,
                                                   int64_t mass_stride, void* stream) {
    using namespace st3;
    st3_status s = check_shape(shape);
    if (s != ST3_OK) return s;
    s = validate_kv(shape, kv, seg);
    if (s != ST3_OK) return s;
    if (!q || !out || !aligned16(q)) return ST3_ERR_INVALID_ARG;
    if (vis_mass && mass_stride < seg->max_vis_len) return ST3_ERR_INVALID_ARG;
    // the scratch is laid out exactly like a caller's workspace for this cache capacity
    const size_t need = decode_ws(shape->batch, shape->heads, shape->head_dim, kv->capacity).total;
    if (need > kScratchBytes) return ST3_ERR_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    s = scratch_for_current_device(&ws);
    if (s != ST3_OK) return s;
    // Nothing in the scratch has to start at zero: the attend launch writes every descriptor, chunk
    // partial and logit that the finish launch of the same call reads.
    return enqueue_decode(shape, q, kv, seg, seg->max_kv_len, nullptr, nullptr, out, vis_mass, mass_stride,
                          vis_mass != nullptr, false, false, ws, kScratchBytes, reinterpret_cast<hipStream_t>(stream));
}
